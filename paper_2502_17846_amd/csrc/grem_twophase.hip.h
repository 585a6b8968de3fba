// Two-phase score path (k <= 16): the same counts as k_score_lds (Alg. 2 cnt_nbrs, Alg. 1 blend,
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
// How: once per call the CSR entries are re-laid-out into 32-bit tuples
// (row_in_slice << cb | column_in_block), grouped by (column block, row chunk):
//   * a column block is 2^cb consecutive vertices counted from the start of their chunk;
//   * a row slice is 2048 consecutive rows counted from the start of their chunk;
//   * segment (c, jb) holds the entries of the rows of chunk c whose column lies in block jb:
//     first the entries of the regular rows, slice by slice, then the entries of the chunk's
//     high-degree rows ("hubs"), share by share (see below).
// T (tuples) is ordered by (jb, c); X (16-bit look-up results, row_in_slice << 5 | valid << 4 |
// label) is ordered by (c, jb); a segment occupies the same number of slots in both, padded to a
// multiple of 8.  After chunk c has been relabelled, k_tp_lookup streams the tuples of c's column
// blocks (contiguous in T), looks the labels up in an LDS copy of the block's labels (two per
// byte) and writes X (contiguous per segment).  Before chunk c is relabelled, k_tp_score has one
// workgroup per row slice gather that slice's sub-segment from every segment (c, *) -- each a few
// hundred bytes, contiguous -- into 16-bit LDS counters, then blends E and proposes.
//
// Balance: rows of degree >= hub_degree are taken out of their slice.  Their entries,
// concatenated in row order, are cut in as many equal shares as the chunk has slices; workgroup i
// of k_tp_score also counts share i (32-bit counters per hub touched) and adds its partial counts
// to a per-chunk table in global memory with integer atomics; k_hub_finalize then blends and
// proposes for the hubs.  The order of entries inside a sub-segment and the order of the atomic
// adds are arbitrary; all of it is integer sums, so the result is not.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "grem_kernels.hip.h"

namespace grem {

constexpr int kSliceRowBits = 11;
constexpr int kSliceRows = 1 << kSliceRowBits;     // rows per slice (row index fits the X entry)
constexpr int kPlanThreads = 256;
constexpr int kTpThreads = 1024;                   // k_tp_lookup and k_tp_score
constexpr int kMaxBlocks = 4096;                   // column blocks (LDS tables in the re-layout kernels)
constexpr int kMaxShareHubs = 2048;                // hubs one share may touch (index fits the X entry)
constexpr int kMaxColBits = 18;                    // 2^18 labels, two per byte: 128 KB of LDS

typedef unsigned long long u64;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct SweepPlan {
    // per slice (global slice index gs = chunk * nsl + i)
    uint32_t *sl_reg_cnt;     // regular (non-hub) entries
    u64 *sl_reg_start;        // their start, relative to the chunk's first entry
    uint32_t *sl_nh;          // hubs in the slice
    uint32_t *sl_hub_start;   // index of the slice's first hub in the chunk's hub list
    u64 *sl_hent;             // hub entries in the slice
    u64 *sl_hent_start;       // their start in the chunk's hub entry stream
    uint32_t *share_h0;       // first hub touched by share gs
    uint32_t *share_nhs;      // hubs touched by share gs
    // per chunk
    u64 *ch_regtot;           // regular entries
    uint32_t *ch_nh;          // hubs
    u64 *ch_H;                // hub entries
    // hub lists: chunk c's hubs at hub_row[chunk_lo + i]; prefix of their degrees at
    // hub_off[chunk_lo + c + i], i = 0..nh (one more slot per chunk)
    int32_t *hub_row;
    u64 *hub_off;
};

// Geometry and offset tables of the re-laid-out entries.
struct TpTables {
    uint32_t *subR;   // [nch * (nsl + 1)][nblk]: start of slice i's regular sub-segment inside segment
                      // (c, jb), row c * (nsl + 1) + i; row i = nsl: end of the regular part
    uint32_t *subH;   // same shape: start of share i's sub-segment; row nsl: end of the segment
    u64 *xstart;      // [nch][nblk] (+1): first slot of segment (c, jb) in X
    u64 *tstart;      // [nblk][nch] (+1): first slot of segment (c, jb) in T
    uint32_t chunk;   // rows per chunk (already clamped to n)
    int chunk_shift;  // log2(chunk) when it is a power of two, else -1
    int nch;          // chunks
    int nsl;          // row slices per chunk
    int nbc;          // column blocks per chunk
    int nblk;         // nch * nbc
    int cb;           // log2 of the vertices per column block
};

__device__ __forceinline__ uint32_t tp_block_of(uint32_t u, const TpTables &g, uint32_t *col_low) {
    const uint32_t cu = g.chunk_shift >= 0 ? (u >> g.chunk_shift) : (u / g.chunk);
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
// plan 1: per slice, regular entries, hubs, hub entries
// ------------------------------------------------------------------------------------------------
template <typename RowT>
__global__ __launch_bounds__(256) void k_plan_slices(const RowT *__restrict__ rowptr, int64_t n,
                                                     int64_t chunk, int nsl, uint32_t hub_degree,
                                                     SweepPlan pl) {
    __shared__ u64 s_reg, s_hent;
    __shared__ uint32_t s_nh;
    const int tid = threadIdx.x;
    const int64_t c = blockIdx.x / nsl;
    const int i = blockIdx.x % nsl;
    const int64_t chunk_lo = c * chunk;
    const int64_t chunk_hi = (chunk_lo + chunk < n) ? chunk_lo + chunk : n;
    const int64_t v0 = chunk_lo + (int64_t)i * kSliceRows;
    if (tid == 0) { s_reg = 0; s_hent = 0; s_nh = 0; }
    __syncthreads();
    u64 reg = 0, hent = 0;
    uint32_t nh = 0;
    for (int q = tid; q < kSliceRows; q += 256) {
        const int64_t v = v0 + q;
        if (v < chunk_hi) {
            const u64 d = (u64)(rowptr[v + 1] - rowptr[v]);
            if (d >= hub_degree) { nh += 1; hent += d; } else reg += d;
        }
    }
    if (reg) atomicAdd(&s_reg, reg);
    if (nh) { atomicAdd(&s_hent, hent); atomicAdd(&s_nh, nh); }
    __syncthreads();
    if (tid == 0) {
        pl.sl_reg_cnt[blockIdx.x] = (uint32_t)s_reg;
        pl.sl_nh[blockIdx.x] = s_nh;
        pl.sl_hent[blockIdx.x] = s_hent;
    }
}

// ------------------------------------------------------------------------------------------------
// plan 2: per chunk, exclusive prefixes over its slices; misc[6] = most hubs in a chunk,
// misc[7] = most entries in a chunk
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_plan_chunks(int64_t n, int64_t chunk, int nsl, SweepPlan pl,
                                                     u64 *__restrict__ misc) {
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
    for (int q = q0; q < q1; ++q) {
        reg += pl.sl_reg_cnt[g0 + q];
        nh += pl.sl_nh[g0 + q];
        hent += pl.sl_hent[g0 + q];
    }
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
        pl.hub_off[chunk_lo + c + bnh] = bhent;
        atomicMax(&misc[6], (u64)bnh);
        atomicMax(&misc[7], breg + bhent);
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
    if (pl.sl_nh[blockIdx.x] == 0) return;
    const int64_t c = blockIdx.x / nsl;
    const int i = blockIdx.x % nsl;
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
            pl.hub_row[chunk_lo + run_nh + ea] = (int32_t)v;
            pl.hub_off[chunk_lo + c + run_nh + ea] = run_ent + eb;
        }
        run_nh += ta;
        run_ent += tb;
    }
}

// ------------------------------------------------------------------------------------------------
// plan 4: per share, the hubs it touches.  Share i of a chunk with NS slices and H hub entries is
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
    if (chunk_lo + (int64_t)i * kSliceRows < chunk_hi) {
        const u64 NS = (u64)((chunk_hi - chunk_lo + kSliceRows - 1) / kSliceRows);
        const u64 H = pl.ch_H[c];
        const u64 a = H * (u64)i / NS, b = H * (u64)(i + 1) / NS;
        if (a != b) {
            const uint32_t nh = pl.ch_nh[c];
            const u64 *goff = pl.hub_off + chunk_lo + c;        // nh + 1 entries, goff[nh] = H
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

// ------------------------------------------------------------------------------------------------
// re-layout of the regular rows of one slice, in two launches of the same kernel:
//   SCATTER = false: count the slice's regular entries per column block -> subR[row(c,i)][*]
//   SCATTER = true : subR now holds sub-segment starts; write the tuples into T
// LDS: rowrel[kSliceRows + 1] (u32) then pos[nblk] (u64, 8-byte aligned)
// ------------------------------------------------------------------------------------------------
template <typename RowT, bool SCATTER>
__global__ __launch_bounds__(256) void k_tp_layout_regular(const RowT *__restrict__ rowptr,
                                                           const int32_t *__restrict__ colidx, int64_t n,
                                                           uint32_t hub_degree, SweepPlan pl, TpTables tb,
                                                           uint32_t *__restrict__ T) {
    extern __shared__ u64 smem64[];
    u64 *pos = smem64;                                                  // nblk
    uint32_t *rowrel = reinterpret_cast<uint32_t *>(pos + tb.nblk);     // kSliceRows + 1
    const int tid = threadIdx.x;
    const int64_t c = blockIdx.x / tb.nsl;
    const int i = blockIdx.x % tb.nsl;
    const int64_t chunk_lo = c * (int64_t)tb.chunk;
    const int64_t chunk_hi = (chunk_lo + tb.chunk < n) ? chunk_lo + tb.chunk : n;
    const int64_t v0 = chunk_lo + (int64_t)i * kSliceRows;
    uint32_t *row_out = tb.subR + ((size_t)c * (tb.nsl + 1) + i) * tb.nblk;
    if (v0 >= chunk_hi) {                       // slice beyond the (ragged) chunk: no entries
        if (!SCATTER) for (int j = tid; j < tb.nblk; j += 256) row_out[j] = 0;
        return;
    }
    const int64_t left = chunk_hi - v0;
    const int nv = left < kSliceRows ? (int)left : kSliceRows;
    const int64_t e0 = (int64_t)rowptr[v0];
    for (int q = tid; q <= kSliceRows; q += 256) {
        int qq = q < nv ? q : nv;
        rowrel[q] = (uint32_t)((int64_t)rowptr[v0 + qq] - e0);
    }
    for (int j = tid; j < tb.nblk; j += 256)
        pos[j] = SCATTER ? tb.tstart[(size_t)j * tb.nch + c] + row_out[j] : 0ull;
    __syncthreads();
    const uint32_t ne = rowrel[kSliceRows];
    const int32_t *cbase = colidx + e0;
    const bool has_hubs = pl.sl_nh[blockIdx.x] != 0;
    for (uint32_t p = tid; p < ne; p += 256) {
        uint32_t r = 0;
        if (SCATTER || has_hubs) {
            r = (uint32_t)owning_row(rowrel, p, kSliceRows);
            if (has_hubs && rowrel[r + 1] - rowrel[r] >= hub_degree) continue;
        }
        uint32_t low;
        const uint32_t jb = tp_block_of((uint32_t)__builtin_nontemporal_load(cbase + p), tb, &low);
        const u64 w = atomicAdd(&pos[jb], 1ull);
        if (SCATTER) T[w] = (r << tb.cb) | low;
    }
    if (!SCATTER) {
        __syncthreads();
        for (int j = tid; j < tb.nblk; j += 256) row_out[j] = (uint32_t)pos[j];
    }
}

// ------------------------------------------------------------------------------------------------
// re-layout of one share of the chunk's hub entries (see k_plan_shares), same two launches; tuples
// carry the hub's index relative to the share's first hub.
// LDS: pos[nblk] (u64), hoff[kMaxShareHubs + 1] (u64), hrow[kMaxShareHubs] (u64)
// ------------------------------------------------------------------------------------------------
template <typename RowT, bool SCATTER>
__global__ __launch_bounds__(256) void k_tp_layout_hubs(const RowT *__restrict__ rowptr,
                                                        const int32_t *__restrict__ colidx, int64_t n,
                                                        SweepPlan pl, TpTables tb, uint32_t *__restrict__ T) {
    extern __shared__ u64 smem64[];
    u64 *pos = smem64;                      // nblk
    u64 *hoff = pos + tb.nblk;              // kMaxShareHubs + 1  stream offsets of the hubs
    u64 *hrow = hoff + kMaxShareHubs + 1;   // kMaxShareHubs      rowptr of the hub
    const int tid = threadIdx.x;
    const int64_t c = blockIdx.x / tb.nsl;
    const int i = blockIdx.x % tb.nsl;
    const int64_t chunk_lo = c * (int64_t)tb.chunk;
    const int64_t chunk_hi = (chunk_lo + tb.chunk < n) ? chunk_lo + tb.chunk : n;
    uint32_t *row_out = tb.subH + ((size_t)c * (tb.nsl + 1) + i) * tb.nblk;
    const bool inside = chunk_lo + (int64_t)i * kSliceRows < chunk_hi;
    const uint32_t h0 = pl.share_h0[blockIdx.x], nhs = pl.share_nhs[blockIdx.x];
    if (!inside || nhs == 0 || nhs > kMaxShareHubs) {      // nothing to do / plan rejected by the host
        if (!SCATTER) for (int j = tid; j < tb.nblk; j += 256) row_out[j] = 0;
        return;
    }
    const u64 NS = (u64)((chunk_hi - chunk_lo + kSliceRows - 1) / kSliceRows);
    const u64 H = pl.ch_H[c];
    const u64 a = H * (u64)i / NS, b = H * (u64)(i + 1) / NS;
    const u64 *goff = pl.hub_off + chunk_lo + c;
    for (int j = tid; j < tb.nblk; j += 256)
        pos[j] = SCATTER ? tb.tstart[(size_t)j * tb.nch + c] + row_out[j] : 0ull;
    for (uint32_t q = tid; q <= nhs; q += 256) hoff[q] = goff[h0 + q];
    for (uint32_t q = tid; q < nhs; q += 256) hrow[q] = (u64)rowptr[pl.hub_row[chunk_lo + h0 + q]];
    __syncthreads();
    const uint32_t len = (uint32_t)(b - a);
    for (uint32_t p = tid; p < len; p += 256) {
        const u64 e = a + p;                                 // position in the chunk's hub entry stream
        uint32_t lo = 0, hi = nhs;
        while (hi - lo > 1) { uint32_t mid = (lo + hi) >> 1; if (hoff[mid] <= e) lo = mid; else hi = mid; }
        const int64_t at = (int64_t)(hrow[lo] + (e - hoff[lo]));
        uint32_t low;
        const uint32_t jb = tp_block_of((uint32_t)__builtin_nontemporal_load(colidx + at), tb, &low);
        const u64 w = atomicAdd(&pos[jb], 1ull);
        if (SCATTER) T[w] = (lo << tb.cb) | low;
    }
    if (!SCATTER) {
        __syncthreads();
        for (int j = tid; j < tb.nblk; j += 256) row_out[j] = (uint32_t)pos[j];
    }
}

// ------------------------------------------------------------------------------------------------
// counts -> starts.  One thread per segment (c, jb): exclusive prefix over the slices of the
// regular counts, then of the share counts; the padded segment length goes to xstart and tstart
// (each in its own order), to be scanned by k_tp_scan_segments.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_tp_scan_slices(TpTables tb) {
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (int64_t)tb.nch * tb.nblk) return;
    const int c = (int)(id / tb.nblk), jb = (int)(id % tb.nblk);
    uint32_t run = 0;
    uint32_t *p = tb.subR + ((size_t)c * (tb.nsl + 1)) * tb.nblk + jb;
    for (int i = 0; i < tb.nsl; ++i, p += tb.nblk) { const uint32_t t = *p; *p = run; run += t; }
    *p = run;
    p = tb.subH + ((size_t)c * (tb.nsl + 1)) * tb.nblk + jb;
    for (int i = 0; i < tb.nsl; ++i, p += tb.nblk) { const uint32_t t = *p; *p = run; run += t; }
    *p = run;
    const u64 padded = ((u64)run + 7ull) & ~7ull;
    tb.xstart[(size_t)c * tb.nblk + jb] = padded;
    tb.tstart[(size_t)jb * tb.nch + c] = padded;
}

// In-place exclusive prefix of a[0..m) by one workgroup, total in a[m].  Block 0 scans xstart,
// block 1 tstart.
__global__ __launch_bounds__(1024) void k_tp_scan_segments(TpTables tb) {
    __shared__ u64 part[1024];
    u64 *a = blockIdx.x == 0 ? tb.xstart : tb.tstart;
    const int64_t m = (int64_t)tb.nch * tb.nblk;
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
// look-up (phase 1 of the score): the tuples of the column blocks of chunk `c0 + blockIdx.y`,
// restricted to row chunks >= cmin, get their labels.  Workgroup blockIdx.x handles share
// (blockIdx.x % spb) of block (blockIdx.x / spb) of the chunk.
//   FROM_LDS = true : the block's labels are copied to LDS, two per byte (every vertex of the
//                     block is assigned: the chunk has just been relabelled)
//   FROM_LDS = false: labels are read from global memory and may be unassigned (valid bit clear);
//                     used once, for the initial labels of a seeded run
// ------------------------------------------------------------------------------------------------
template <bool FROM_LDS>
__global__ __launch_bounds__(kTpThreads) void k_tp_lookup(const uint32_t *__restrict__ T,
                                                          uint16_t *__restrict__ X, TpTables tb,
                                                          const uint8_t *__restrict__ Lc, int64_t n, int c0,
                                                          int cmin, int spb) {
    extern __shared__ uint32_t tab[];      // 2^cb / 8 words (FROM_LDS)
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
    const u64 units = (hi - lo) >> 3;
    const u64 p0 = lo + ((units * (u64)s / (u64)spb) << 3);
    const u64 p1 = lo + ((units * (u64)(s + 1) / (u64)spb) << 3);
    if (p0 >= p1) return;

    if (FROM_LDS) {
        const int64_t bv = (chunk_hi - block_lo) < (1ll << tb.cb) ? (chunk_hi - block_lo) : (1ll << tb.cb);
        const int words = (int)((bv + 7) >> 3);
        const uint8_t *src = Lc + block_lo;
        const bool aligned = (((uintptr_t)src) & 7u) == 0;
        for (int w = tid; w < words; w += kTpThreads) {
            uint32_t packed = 0;
            if (aligned && (int64_t)w * 8 + 8 <= bv) {
                const u32x2 v = *reinterpret_cast<const u32x2 *>(src + (size_t)w * 8);
                const uint32_t a = v.x, b = v.y;
                const uint32_t p = (a & 15u) | ((a >> 4) & 0xF0u) | ((a >> 8) & 0xF00u) | ((a >> 12) & 0xF000u);
                const uint32_t q = (b & 15u) | ((b >> 4) & 0xF0u) | ((b >> 8) & 0xF00u) | ((b >> 12) & 0xF000u);
                packed = p | (q << 16);
            } else {
                for (int q = 0; q < 8; ++q) {
                    const int64_t o = (int64_t)w * 8 + q;
                    if (o < bv) packed |= ((uint32_t)src[o] & 15u) << (4 * q);
                }
            }
            tab[w] = packed;
        }
        __syncthreads();
    }
    const uint8_t *tbytes = reinterpret_cast<const uint8_t *>(tab);
    const uint32_t cmask = (1u << tb.cb) - 1u;

    // first row chunk whose segment ends after p0
    int cc = cmin;
    {
        int a = cmin, b = tb.nch - 1;       // ts[b + 1] = hi > p0 always holds
        while (a < b) { const int mid = (a + b) >> 1; if (ts[mid + 1] > p0) b = mid; else a = mid + 1; }
        cc = a;
    }
    u64 p = p0;
    while (p < p1 && cc < tb.nch) {
        const u64 seg_lo = ts[cc], seg_hi = ts[cc + 1];
        const u64 e = seg_hi < p1 ? seg_hi : p1;
        if (e > p) {
            const u64 xp = tb.xstart[(size_t)cc * tb.nblk + jb] + (p - seg_lo);
            const u32x4 *src4 = reinterpret_cast<const u32x4 *>(T + p);
            u32x2 *dst2 = reinterpret_cast<u32x2 *>(X + xp);
            const uint32_t ng = (uint32_t)((e - p) >> 2);
            constexpr int U = 2;
            for (uint32_t base = tid; base < ng; base += kTpThreads * U) {
                u32x4 t[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint32_t g = base + u * kTpThreads;
                    t[u] = g < ng ? __builtin_nontemporal_load(src4 + g) : (u32x4)(0u);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint32_t g = base + u * kTpThreads;
                    if (g < ng) {
                        const uint32_t ent[4] = {t[u].x, t[u].y, t[u].z, t[u].w};
                        uint32_t o[4];
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const uint32_t col = ent[q] & cmask;
                            uint32_t lab;
                            if (FROM_LDS) {
                                lab = 16u | (((uint32_t)tbytes[col >> 1] >> (4 * (col & 1u))) & 15u);
                            } else {
                                const int64_t v = block_lo + (int64_t)col;
                                const uint32_t l = v < chunk_hi ? (uint32_t)Lc[v] : 0xFFu;
                                lab = l == 0xFFu ? 0u : (16u | (l & 15u));
                            }
                            o[q] = (((ent[q] >> tb.cb) << 5) | lab) & 0xFFFFu;
                        }
                        u32x2 w;
                        w.x = o[0] | (o[1] << 16);
                        w.y = o[2] | (o[3] << 16);
                        __builtin_nontemporal_store(w, dst2 + g);
                    }
                }
            }
            p = e;
        }
        cc += 1;
    }
}

// one 16-bit look-up result into the counters; COUNT16: two 16-bit counters per word, else 32-bit
template <bool COUNT16>
__device__ __forceinline__ void tp_count_entry(uint32_t x, int k, uint32_t *hist) {
    if (x & 16u) {
        const uint32_t c = (x >> 5) * (uint32_t)k + (x & 15u);
        if (COUNT16) atomicAdd(&hist[c >> 1], 1u << (16 * (c & 1u)));
        else atomicAdd(&hist[c], 1u);
    }
}

// two sub-segments [sa, ea) and [sb, eb) of X, taken together by one wavefront so that the loads
// of both are in flight at once
template <bool COUNT16, int U>
__device__ __forceinline__ void tp_count_pair(const uint16_t *__restrict__ X, u64 sa, u64 ea, u64 sb,
                                              u64 eb, int lane, int k, uint32_t *hist) {
    uint32_t va[U], vb[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const u64 qa = sa + (u64)(lane + 64 * u), qb = sb + (u64)(lane + 64 * u);
        va[u] = qa < ea ? (uint32_t)__builtin_nontemporal_load(X + qa) : 0u;
        vb[u] = qb < eb ? (uint32_t)__builtin_nontemporal_load(X + qb) : 0u;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        tp_count_entry<COUNT16>(va[u], k, hist);
        tp_count_entry<COUNT16>(vb[u], k, hist);
    }
    for (u64 q = sa + (u64)(lane + 64 * U); q < ea; q += 64)
        tp_count_entry<COUNT16>((uint32_t)__builtin_nontemporal_load(X + q), k, hist);
    for (u64 q = sb + (u64)(lane + 64 * U); q < eb; q += 64)
        tp_count_entry<COUNT16>((uint32_t)__builtin_nontemporal_load(X + q), k, hist);
}

// ------------------------------------------------------------------------------------------------
// score (phase 2): one workgroup per row slice of chunk c, plus one share of the chunk's hub
// entries.  Column blocks [0, jlim) are counted (in the first pass of an unseeded run the blocks of
// chunks >= c hold no label yet and their part of X has not been written).
// ------------------------------------------------------------------------------------------------
template <typename RowT>
__global__ __launch_bounds__(kTpThreads) void k_tp_score(
    const RowT *__restrict__ rowptr, const uint16_t *__restrict__ X, TpTables tb, SweepPlan pl,
    const uint8_t *__restrict__ Lc, const long long *__restrict__ S, uint32_t *__restrict__ E,
    uint32_t *__restrict__ Hhub, uint8_t *__restrict__ prop, int c, int64_t chunk_lo, int64_t chunk_hi,
    int k, int jlim, int share_hubs, uint32_t hub_degree, int pass, long long P) {
    extern __shared__ uint32_t smem[];
    const int hist_words = (kSliceRows * k + 1) >> 1;
    uint32_t *hist = smem;                      // hist_words            regular rows, 16-bit counters
    uint32_t *hhist = hist + hist_words;        // share_hubs * k        hubs of the share, 32-bit
    uint32_t *room = hhist + share_hubs * k;    // k
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    constexpr int NW = kTpThreads / 64;
    const size_t gs = (size_t)c * tb.nsl + blockIdx.x;
    const int64_t v0 = chunk_lo + (int64_t)blockIdx.x * kSliceRows;
    const int64_t left = chunk_hi - v0;
    const int nv = left < kSliceRows ? (int)left : kSliceRows;

    for (int q = tid; q < hist_words + share_hubs * k; q += kTpThreads) hist[q] = 0;
    for (int j = tid; j < k; j += kTpThreads) room[j] = (uint32_t)(P - S[j]);
    __syncthreads();

    const bool any_hub = pl.share_nhs[gs] != 0;
    const uint32_t *r0 = tb.subR + ((size_t)c * (tb.nsl + 1) + blockIdx.x) * tb.nblk;
    const uint32_t *r1 = r0 + tb.nblk;
    const uint32_t *q0 = tb.subH + ((size_t)c * (tb.nsl + 1) + blockIdx.x) * tb.nblk;
    const uint32_t *q1 = q0 + tb.nblk;
    const u64 *xs = tb.xstart + (size_t)c * tb.nblk;
    for (int base = 0; base < jlim; base += NW * 64) {
        // lane l of wave w holds the offsets of block base + w + NW * l
        const int jl = base + wave + NW * lane;
        u64 x0 = 0;
        uint32_t a0 = 0, a1 = 0, h0 = 0, h1 = 0;
        if (jl < jlim) {
            x0 = xs[jl];
            a0 = r0[jl];
            a1 = r1[jl];
            if (any_hub) { h0 = q0[jl]; h1 = q1[jl]; }
        }
        int tmax = (jlim - base - wave + NW - 1) / NW;      // blocks of this wave in this round
        if (tmax > 64) tmax = 64;
        for (int t = 0; t < tmax; t += 2) {
            const int t2 = t + 1 < tmax ? t + 1 : t;
            const u64 xa = __shfl(x0, t), xb = __shfl(x0, t2);
            const uint32_t sa = __shfl(a0, t), ea = __shfl(a1, t);
            const uint32_t sb = __shfl(a0, t2), eb = t2 != t ? __shfl(a1, t2) : sb;
            tp_count_pair<true, 3>(X, xa + sa, xa + ea, xb + sb, xb + eb, lane, k, hist);
        }
        if (any_hub) {
            for (int t = 0; t < tmax; t += 2) {
                const int t2 = t + 1 < tmax ? t + 1 : t;
                const u64 xa = __shfl(x0, t), xb = __shfl(x0, t2);
                const uint32_t sa = __shfl(h0, t), ea = __shfl(h1, t);
                const uint32_t sb = __shfl(h0, t2), eb = t2 != t ? __shfl(h1, t2) : sb;
                tp_count_pair<false, 1>(X, xa + sa, xa + ea, xb + sb, xb + eb, lane, k, hhist);
            }
        }
    }
    __syncthreads();

    // partial counts of the share's hubs -> the chunk's hub table
    if (any_hub) {
        const uint32_t h0 = pl.share_h0[gs];
        for (int q = tid; q < share_hubs * k; q += kTpThreads) {
            const uint32_t x = hhist[q];
            if (x) atomicAdd(&Hhub[(size_t)h0 * k + q], x);
        }
    }

    // blend and propose: four lanes per regular vertex, lane q takes partitions q*4.. (k % 4 == 0)
    // or q, q+4, .. (otherwise); arg-max by (E desc, room desc, id asc)
    const int sh = pass > 0 ? pass - 1 : 0;
    for (int g = tid; g < nv * 4; g += kTpThreads) {
        const int t = g >> 2, q = g & 3;
        const int64_t v = v0 + t;
        if ((u64)(rowptr[v + 1] - rowptr[v]) >= hub_degree) continue;      // k_hub_finalize's
        const uint32_t old = (uint32_t)Lc[v];
        uint32_t *Erow = E + (size_t)v * (size_t)k;
        unsigned long long bestkey = 0;
        int bestj = 0x7fffffff;
        const uint32_t cbase = (uint32_t)t * (uint32_t)k;
        if ((k & 3) == 0) {
            for (int j4 = q * 4; j4 < k; j4 += 16) {
                u32x4 e = (u32x4)(0u);
                if (pass > 0) e = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(Erow + j4));
                const uint32_t w0 = hist[(cbase + j4) >> 1], w1 = hist[((cbase + j4) >> 1) + 1];
                const uint32_t ev[4] = {e.x + ((w0 & 0xFFFFu) << sh), e.y + ((w0 >> 16) << sh),
                                        e.z + ((w1 & 0xFFFFu) << sh), e.w + ((w1 >> 16) << sh)};
                u32x4 o;
                o.x = ev[0]; o.y = ev[1]; o.z = ev[2]; o.w = ev[3];
                __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(Erow + j4));
#pragma unroll
                for (int z = 0; z < 4; ++z) {
                    const int j = j4 + z;
                    const uint32_t rm = room[j] + ((uint32_t)j == old ? 1u : 0u);
                    const unsigned long long key = rm ? (((unsigned long long)ev[z] << 32) | rm) : 0ull;
                    if (key > bestkey) { bestkey = key; bestj = j; }
                }
            }
        } else {
            for (int j = q; j < k; j += 4) {
                const uint32_t cidx = cbase + (uint32_t)j;
                const uint32_t h = (hist[cidx >> 1] >> (16 * (cidx & 1u))) & 0xFFFFu;
                const uint32_t e = (pass > 0 ? Erow[j] : 0u) + (h << sh);
                Erow[j] = e;
                const uint32_t rm = room[j] + ((uint32_t)j == old ? 1u : 0u);
                const unsigned long long key = rm ? (((unsigned long long)e << 32) | rm) : 0ull;
                if (key > bestkey) { bestkey = key; bestj = j; }
            }
        }
#pragma unroll
        for (int off = 1; off <= 2; off <<= 1) {
            const unsigned long long okey = __shfl_xor(bestkey, off);
            const int oj = __shfl_xor(bestj, off);
            if (okey > bestkey || (okey == bestkey && oj < bestj)) { bestkey = okey; bestj = oj; }
        }
        if (q == 0) {
            uint32_t best = (uint32_t)bestj;
            if (pass == 0 && old != 0xFFu) best = old;      // seeded vertex keeps its label
            prop[v - chunk_lo] = (uint8_t)best;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// hubs of the chunk: counts from the hub table (complete once k_tp_score has finished), blend,
// propose; the table row is cleared for the next chunk.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_hub_finalize(SweepPlan pl, const uint8_t *__restrict__ Lc,
                                                      const long long *__restrict__ S,
                                                      uint32_t *__restrict__ E, uint32_t *__restrict__ Hhub,
                                                      uint8_t *__restrict__ prop, int64_t chunk_idx,
                                                      int64_t chunk_lo, int k, int pass, long long P) {
    const uint32_t nh = pl.ch_nh[chunk_idx];
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nh) return;
    const int64_t v = pl.hub_row[chunk_lo + i];
    const uint32_t old = (uint32_t)Lc[v];
    uint32_t *Erow = E + (size_t)v * (size_t)k;
    uint32_t *hrow = Hhub + (size_t)i * k;
    const int sh = pass > 0 ? pass - 1 : 0;
    unsigned long long bestkey = 0;
    int bestj = 0x7fffffff;
    for (int j = 0; j < k; ++j) {
        const uint32_t h = hrow[j];
        hrow[j] = 0;
        const uint32_t e = (pass > 0 ? Erow[j] : 0u) + (h << sh);
        Erow[j] = e;
        const long long rml = P - S[j] + ((uint32_t)j == old ? 1 : 0);
        const uint32_t rm = (uint32_t)rml;
        unsigned long long key = rm ? (((unsigned long long)e << 32) | rm) : 0ull;
        if (key > bestkey) { bestkey = key; bestj = j; }
    }
    uint32_t best = (uint32_t)bestj;
    if (pass == 0 && old != 0xFFu) best = old;
    prop[v - chunk_lo] = (uint8_t)best;
}

}  // namespace grem
