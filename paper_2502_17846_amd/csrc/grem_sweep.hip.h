// Column-sliced score path (k <= 16): the same counts as k_score_lds (Alg. 2 cnt_nbrs, Alg. 1
// blend, Alg. 2 assign), organised so that the neighbour-label look-ups hit L2.
//
// Why: a look-up into a label table larger than L2 costs one 64-byte fabric request whatever the
// table's size (57 G/s on MI355X), while look-ups into an L2-resident table run at 267 G/s.
//
// How: once per call the CSR entries are re-laid-out.  A chunk's rows are grouped in slices of 2048
// consecutive rows; a score workgroup owns one slice, keeps its histograms in LDS as 16-bit
// counters and walks its entries bucket by bucket in ascending column slice (col >> col_bits).
// All workgroups of a chunk are resident together and start together, so at any moment they read
// the same one or two column slices of the label table (1 MB each with two labels per byte), which
// therefore stay in each XCD's L2.  Entries are stored as 32-bit tuples
// (row_in_slice << col_bits | col_low).
//
// Balance: a chunk's kernel lasts as long as its slowest workgroup, so rows of degree >= hub_degree
// ("hubs") are taken out of their slice.  Their entries, concatenated in row order, are cut in as
// many equal shares as the chunk has slices; workgroup i also processes share i (bucketed the same
// way, 32-bit counters per hub touched) and adds its partial counts to a per-chunk table in global
// memory with integer atomics; k_hub_finalize then blends and proposes for the hubs.  The order of
// entries inside a bucket and the order of the atomic adds are arbitrary; all of it is integer
// sums, so the result is not.
//
// Layout of tup for chunk c (eb = rowptr[chunk_lo]):  [slice 0 regular | slice 1 regular | ... |
// share 0 | share 1 | ...], regular part of slice s at eb + sl_reg_start[s], share i at
// eb + ch_regtot[c] + H_c * i / NS_c  (H_c hub entries, NS_c slices of the chunk).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "grem_kernels.hip.h"

namespace grem {

constexpr int kSliceRowBits = 11;
constexpr int kSliceRows = 1 << kSliceRowBits;     // rows per slice (row index fits the tuple)
constexpr int kSweepThreads = 256;
constexpr int kMaxColSlices = 2048;                // LDS tables in the relayout kernels
constexpr int kMaxShareHubs = 2048;                // hubs one share may touch (LDS table in relayout)

typedef unsigned long long u64;

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
    for (int w = 0; w < kSweepThreads / 64; ++w) {
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
// plan 2: per chunk, exclusive prefixes over its slices; misc[6] = most hubs in a chunk
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
// relayout of the regular rows of one slice: counting sort of their entries by column slice.
//   boff[gs][j] first tuple of column slice j (relative to the slice's start), boff[gs][ncs] total
// ------------------------------------------------------------------------------------------------
template <typename RowT>
__global__ __launch_bounds__(256) void k_relayout_regular(const RowT *__restrict__ rowptr,
                                                          const int32_t *__restrict__ colidx, int64_t n,
                                                          int64_t chunk, int nsl, int ncs, int col_bits,
                                                          uint32_t hub_degree, SweepPlan pl,
                                                          uint32_t *__restrict__ tup,
                                                          uint32_t *__restrict__ boff) {
    extern __shared__ uint32_t smem[];
    uint32_t *rowrel = smem;                    // kSliceRows + 1
    uint32_t *cnt = rowrel + kSliceRows + 1;    // ncs
    const int tid = threadIdx.x;
    const int64_t c = blockIdx.x / nsl;
    const int i = blockIdx.x % nsl;
    const int64_t chunk_lo = c * chunk;
    const int64_t chunk_hi = (chunk_lo + chunk < n) ? chunk_lo + chunk : n;
    const int64_t v0 = chunk_lo + (int64_t)i * kSliceRows;
    if (v0 >= chunk_hi) return;
    const int64_t left = chunk_hi - v0;
    const int nv = left < kSliceRows ? (int)left : kSliceRows;
    const int64_t e0 = (int64_t)rowptr[v0];
    for (int q = tid; q <= kSliceRows; q += 256) {
        int qq = q < nv ? q : nv;
        rowrel[q] = (uint32_t)((int64_t)rowptr[v0 + qq] - e0);
    }
    for (int j = tid; j < ncs; j += 256) cnt[j] = 0;
    __syncthreads();
    const uint32_t ne = rowrel[kSliceRows];
    const int32_t *cbase = colidx + e0;
    const bool has_hubs = pl.sl_nh[blockIdx.x] != 0;
    for (uint32_t p = tid; p < ne; p += 256) {
        if (has_hubs) {
            const int r = owning_row(rowrel, p, kSliceRows);
            if (rowrel[r + 1] - rowrel[r] >= hub_degree) continue;
        }
        atomicAdd(&cnt[(uint32_t)cbase[p] >> col_bits], 1u);
    }
    __syncthreads();
    uint32_t *bo = boff + (size_t)blockIdx.x * (ncs + 1);
    if (tid == 0) {
        uint32_t run = 0;
        for (int j = 0; j < ncs; ++j) {
            uint32_t cj = cnt[j];
            cnt[j] = run;          // becomes the bucket's write cursor
            bo[j] = run;
            run += cj;
        }
        bo[ncs] = run;
    }
    __syncthreads();
    const uint32_t mask = (1u << col_bits) - 1u;
    uint32_t *tbase = tup + (int64_t)rowptr[chunk_lo] + (int64_t)pl.sl_reg_start[blockIdx.x];
    for (uint32_t p = tid; p < ne; p += 256) {
        const uint32_t r = (uint32_t)owning_row(rowrel, p, kSliceRows);
        if (has_hubs && rowrel[r + 1] - rowrel[r] >= hub_degree) continue;
        const uint32_t col = (uint32_t)cbase[p];
        const uint32_t pos = atomicAdd(&cnt[col >> col_bits], 1u);
        tbase[pos] = (r << col_bits) | (col & mask);
    }
}

// ------------------------------------------------------------------------------------------------
// relayout of one share of the chunk's hub entries (see k_plan_shares); tuples carry the hub's index
// relative to the share's first hub.  hboff[gs][.] as boff.
// ------------------------------------------------------------------------------------------------
template <typename RowT>
__global__ __launch_bounds__(256) void k_relayout_hubs(const RowT *__restrict__ rowptr,
                                                       const int32_t *__restrict__ colidx, int64_t n,
                                                       int64_t chunk, int nsl, int ncs, int col_bits,
                                                       SweepPlan pl, uint32_t *__restrict__ tup,
                                                       uint32_t *__restrict__ hboff) {
    extern __shared__ uint32_t smem[];
    uint32_t *cnt = smem;                                   // ncs
    u64 *hoff = (u64 *)(smem + ((ncs + 1) & ~1));          // kMaxShareHubs + 1  stream offsets of the hubs
    u64 *hrow = hoff + kMaxShareHubs + 1;                   // kMaxShareHubs      rowptr of the hub
    const int tid = threadIdx.x;
    const int64_t c = blockIdx.x / nsl;
    const int i = blockIdx.x % nsl;
    const int64_t chunk_lo = c * chunk;
    const int64_t chunk_hi = (chunk_lo + chunk < n) ? chunk_lo + chunk : n;
    if (chunk_lo + (int64_t)i * kSliceRows >= chunk_hi) return;
    uint32_t *bo = hboff + (size_t)blockIdx.x * (ncs + 1);
    const uint32_t h0 = pl.share_h0[blockIdx.x], nhs = pl.share_nhs[blockIdx.x];
    if (nhs == 0 || nhs > kMaxShareHubs) {      // nothing to do / plan rejected by the host
        for (int j = tid; j <= ncs; j += 256) bo[j] = 0;
        return;
    }
    const u64 NS = (u64)((chunk_hi - chunk_lo + kSliceRows - 1) / kSliceRows);
    const u64 H = pl.ch_H[c];
    const u64 a = H * (u64)i / NS, b = H * (u64)(i + 1) / NS;
    const u64 *goff = pl.hub_off + chunk_lo + c;
    for (int j = tid; j < ncs; j += 256) cnt[j] = 0;
    for (uint32_t q = tid; q <= nhs; q += 256) hoff[q] = goff[h0 + q];
    for (uint32_t q = tid; q < nhs; q += 256) hrow[q] = (u64)rowptr[pl.hub_row[chunk_lo + h0 + q]];
    __syncthreads();
    const uint32_t len = (uint32_t)(b - a);
    auto locate = [&](u64 e, uint32_t *hl) -> int64_t {     // hub and colidx position of stream entry e
        uint32_t lo = 0, hi = nhs;
        while (hi - lo > 1) { uint32_t mid = (lo + hi) >> 1; if (hoff[mid] <= e) lo = mid; else hi = mid; }
        *hl = lo;
        return (int64_t)(hrow[lo] + (e - hoff[lo]));
    };
    for (uint32_t p = tid; p < len; p += 256) {
        uint32_t hl;
        const int64_t pos = locate(a + p, &hl);
        atomicAdd(&cnt[(uint32_t)colidx[pos] >> col_bits], 1u);
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t run = 0;
        for (int j = 0; j < ncs; ++j) { uint32_t cj = cnt[j]; cnt[j] = run; bo[j] = run; run += cj; }
        bo[ncs] = run;
    }
    __syncthreads();
    const uint32_t mask = (1u << col_bits) - 1u;
    uint32_t *tbase = tup + (int64_t)rowptr[chunk_lo] + (int64_t)pl.ch_regtot[c] + (int64_t)a;
    for (uint32_t p = tid; p < len; p += 256) {
        uint32_t hl;
        const int64_t pos = locate(a + p, &hl);
        const uint32_t col = (uint32_t)colidx[pos];
        const uint32_t w = atomicAdd(&cnt[col >> col_bits], 1u);
        tbase[w] = (hl << col_bits) | (col & mask);
    }
}

// ------------------------------------------------------------------------------------------------
// pack: two labels per byte for rows [lo, hi) (whole bytes; the neighbour of a boundary row is
// re-packed with it).  Unassigned labels pack to 0xF and are never looked up.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_pack(const uint8_t *__restrict__ Lc, uint8_t *__restrict__ Ln,
                                              int64_t lo, int64_t hi, int64_t n) {
    const int64_t b0 = lo >> 1, b1 = (hi + 1) >> 1;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t b = b0 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; b < b1; b += stride) {
        const int64_t v = b << 1;
        uint32_t x = Lc[v] & 15u;
        uint32_t y = (v + 1 < n) ? (Lc[v + 1] & 15u) : 0u;
        Ln[b] = (uint8_t)(x | (y << 4));
    }
}

// one bucket: tuples [b0, b1) of tbase; COUNT16: 16-bit counters packed two per word, else 32-bit
template <bool NIB, bool COUNT16>
__device__ __forceinline__ void sweep_bucket(const uint32_t *__restrict__ tbase, uint32_t b0, uint32_t b1,
                                             int64_t cb, uint32_t mask, int col_bits, int k,
                                             int64_t gather_limit, const uint8_t *__restrict__ Lc,
                                             const uint8_t *__restrict__ Ln, uint32_t *hist) {
    constexpr int U = 4;
    for (uint32_t base = b0 + threadIdx.x; base < b1; base += kSweepThreads * U) {
        uint32_t t[U], lab[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint32_t p = base + u * kSweepThreads;
            t[u] = (p < b1) ? __builtin_nontemporal_load(tbase + p) : 0xFFFFFFFFu;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            lab[u] = 0xFFu;
            const int64_t col = cb | (int64_t)(t[u] & mask);
            if (t[u] != 0xFFFFFFFFu && col < gather_limit) {
                if (NIB) lab[u] = ((uint32_t)Ln[col >> 1] >> (4 * (int)(col & 1))) & 15u;
                else lab[u] = Lc[col];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (lab[u] != 0xFFu) {
                const uint32_t c = (t[u] >> col_bits) * (uint32_t)k + lab[u];
                if (COUNT16) atomicAdd(&hist[c >> 1], 1u << (16 * (c & 1u)));
                else atomicAdd(&hist[c], 1u);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// score over one row slice plus one share of the chunk's hub entries.
// NIB: labels are read from the packed table Ln (valid when no looked-up vertex is unassigned:
// every pass of an unseeded run, and passes >= 1 of any run); otherwise from Lc.
// ------------------------------------------------------------------------------------------------
template <typename RowT, bool NIB>
__global__ __launch_bounds__(kSweepThreads) void k_score_sweep(
    const RowT *__restrict__ rowptr, const uint32_t *__restrict__ tup,
    const uint32_t *__restrict__ boff, const uint32_t *__restrict__ hboff, SweepPlan pl,
    const uint8_t *__restrict__ Lc, const uint8_t *__restrict__ Ln, const long long *__restrict__ S,
    uint32_t *__restrict__ E, uint32_t *__restrict__ Hhub, uint8_t *__restrict__ prop, int64_t chunk_idx,
    int64_t chunk_lo, int64_t chunk_hi, int nsl, int k, int ncs, int col_bits, int share_hubs,
    uint32_t hub_degree, int pass, long long P, int64_t gather_limit) {
    extern __shared__ uint32_t smem[];
    const int hist_words = (kSliceRows * k + 1) >> 1;
    uint32_t *hist = smem;                      // hist_words            regular rows, 16-bit counters
    uint32_t *hhist = hist + hist_words;        // share_hubs * k        hubs of the share, 32-bit
    uint32_t *bo = hhist + share_hubs * k;      // ncs + 1
    uint32_t *hbo = bo + ncs + 1;               // ncs + 1
    uint32_t *room = hbo + ncs + 1;             // k
    const int tid = threadIdx.x;
    const size_t gs = (size_t)chunk_idx * nsl + blockIdx.x;
    const int64_t v0 = chunk_lo + (int64_t)blockIdx.x * kSliceRows;
    const int64_t left = chunk_hi - v0;
    const int nv = left < kSliceRows ? (int)left : kSliceRows;
    const uint32_t *gbo = boff + gs * (ncs + 1);
    const uint32_t *ghbo = hboff + gs * (ncs + 1);

    for (int q = tid; q < hist_words + share_hubs * k; q += kSweepThreads) hist[q] = 0;
    for (int q = tid; q <= ncs; q += kSweepThreads) { bo[q] = gbo[q]; hbo[q] = ghbo[q]; }
    for (int j = tid; j < k; j += kSweepThreads) room[j] = (uint32_t)(P - S[j]);
    __syncthreads();

    const int64_t eb = (int64_t)rowptr[chunk_lo];
    const u64 NS = (u64)((chunk_hi - chunk_lo + kSliceRows - 1) / kSliceRows);
    const u64 H = pl.ch_H[chunk_idx];
    const uint32_t *tbase = tup + eb + (int64_t)pl.sl_reg_start[gs];
    const uint32_t *htbase = tup + eb + (int64_t)pl.ch_regtot[chunk_idx] + (int64_t)(H * (u64)blockIdx.x / NS);
    const uint32_t mask = (1u << col_bits) - 1u;
    const bool any_hub = hbo[ncs] != 0;
    for (int j = 0; j < ncs; ++j) {
        const int64_t cb = (int64_t)j << col_bits;
        if (cb >= gather_limit) break;
        sweep_bucket<NIB, true>(tbase, bo[j], bo[j + 1], cb, mask, col_bits, k, gather_limit, Lc, Ln, hist);
        if (any_hub)
            sweep_bucket<NIB, false>(htbase, hbo[j], hbo[j + 1], cb, mask, col_bits, k, gather_limit, Lc, Ln,
                                     hhist);
    }
    __syncthreads();

    // partial counts of the share's hubs -> the chunk's hub table
    if (any_hub) {
        const uint32_t h0 = pl.share_h0[gs];
        for (int q = tid; q < share_hubs * k; q += kSweepThreads) {
            const uint32_t x = hhist[q];
            if (x) atomicAdd(&Hhub[(size_t)h0 * k + q], x);
        }
    }

    // blend and propose, one thread per regular vertex
    const int sh = pass > 0 ? pass - 1 : 0;
    for (int t = tid; t < nv; t += kSweepThreads) {
        const int64_t v = v0 + t;
        if ((u64)(rowptr[v + 1] - rowptr[v]) >= hub_degree) continue;      // k_hub_finalize's
        const uint32_t old = (uint32_t)Lc[v];
        uint32_t *Erow = E + (size_t)v * (size_t)k;
        unsigned long long bestkey = 0;
        int bestj = 0x7fffffff;
        const uint32_t cbase = (uint32_t)t * (uint32_t)k;
        if ((k & 3) == 0) {
            for (int j4 = 0; j4 < k; j4 += 4) {
                uint4 e = make_uint4(0, 0, 0, 0);
                if (pass > 0) e = *reinterpret_cast<const uint4 *>(Erow + j4);
                const uint32_t w0 = hist[(cbase + j4) >> 1], w1 = hist[((cbase + j4) >> 1) + 1];
                uint32_t ev[4] = {e.x + ((w0 & 0xFFFFu) << sh), e.y + ((w0 >> 16) << sh),
                                  e.z + ((w1 & 0xFFFFu) << sh), e.w + ((w1 >> 16) << sh)};
                *reinterpret_cast<uint4 *>(Erow + j4) = make_uint4(ev[0], ev[1], ev[2], ev[3]);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int j = j4 + q;
                    uint32_t rm = room[j] + ((uint32_t)j == old ? 1u : 0u);
                    unsigned long long key = rm ? (((unsigned long long)ev[q] << 32) | rm) : 0ull;
                    if (key > bestkey) { bestkey = key; bestj = j; }
                }
            }
        } else {
            for (int j = 0; j < k; ++j) {
                const uint32_t c = cbase + (uint32_t)j;
                const uint32_t h = (hist[c >> 1] >> (16 * (c & 1u))) & 0xFFFFu;
                const uint32_t e = (pass > 0 ? Erow[j] : 0u) + (h << sh);
                Erow[j] = e;
                uint32_t rm = room[j] + ((uint32_t)j == old ? 1u : 0u);
                unsigned long long key = rm ? (((unsigned long long)e << 32) | rm) : 0ull;
                if (key > bestkey) { bestkey = key; bestj = j; }
            }
        }
        uint32_t best = (uint32_t)bestj;
        if (pass == 0 && old != 0xFFu) best = old;      // seeded vertex keeps its label
        prop[v - chunk_lo] = (uint8_t)best;
    }
}

// ------------------------------------------------------------------------------------------------
// hubs of the chunk: counts from the hub table (complete once k_score_sweep has finished), blend,
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
