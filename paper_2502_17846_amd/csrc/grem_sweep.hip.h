// Column-sliced score path (k <= 16): the same counts as k_score_lds (Alg. 2 cnt_nbrs, Alg. 1
// blend, Alg. 2 assign), organised so that the neighbour-label look-ups hit L2.
//
// Why: a look-up into a label table larger than L2 costs one 64-byte fabric request whatever the
// table's size (57 G/s on MI355X), while look-ups into an L2-resident table run at 267 G/s.
//
// How: once per call the CSR entries are re-laid-out (k_relayout).  Rows are grouped in slices of
// up to 2048 consecutive rows; inside a slice the entries are bucketed by column slice
// (col >> col_bits) and stored as 32-bit tuples (row_in_slice << col_bits | col_low).  A score
// workgroup owns one row slice, keeps its histograms in LDS as 16-bit counters and walks its
// buckets in ascending column slice.  All workgroups of a chunk are resident together and start
// together, so at any moment they read the same one or two column slices of the label table
// (1 MB each with labels packed two per byte), which therefore stay in each XCD's L2.  The order
// of entries inside a bucket is arbitrary; counts are integer sums, so the result is not.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "grem_kernels.hip.h"

namespace grem {

constexpr int kSliceRowBits = 11;
constexpr int kSliceRows = 1 << kSliceRowBits;     // rows per slice (row index fits the tuple)
constexpr int kSweepThreads = 256;
constexpr int kMaxColSlices = 2048;                // LDS tables in k_relayout

// ------------------------------------------------------------------------------------------------
// relayout: one workgroup per row slice; counting sort of the slice's entries by column slice.
//   tup[rowptr[v0] + p]  p-th tuple of the slice, buckets in ascending column slice
//   boff[slice][j]       first tuple of column slice j (relative), boff[slice][ncs] = slice entries
// Slices are numbered chunk_index * nsl + i (i-th group of 2048 rows of the chunk).
// ------------------------------------------------------------------------------------------------
template <typename RowT>
__global__ __launch_bounds__(256) void k_relayout(const RowT *__restrict__ rowptr,
                                                  const int32_t *__restrict__ colidx, int64_t n,
                                                  int64_t chunk, int nsl, int ncs, int col_bits,
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
    for (uint32_t p = tid; p < ne; p += 256) atomicAdd(&cnt[(uint32_t)cbase[p] >> col_bits], 1u);
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
    uint32_t *tbase = tup + e0;
    for (uint32_t p = tid; p < ne; p += 256) {
        const uint32_t col = (uint32_t)cbase[p];
        const uint32_t r = (uint32_t)owning_row(rowrel, p, kSliceRows);
        const uint32_t pos = atomicAdd(&cnt[col >> col_bits], 1u);
        tbase[pos] = (r << col_bits) | (col & mask);
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

// ------------------------------------------------------------------------------------------------
// score over one row slice.  hist: 16-bit counters, two per LDS word, index row * k + label.
// NIB: labels are read from the packed table Ln (valid when no looked-up vertex is unassigned:
// every pass of an unseeded run, and passes >= 1 of any run); otherwise from Lc.
// ------------------------------------------------------------------------------------------------
template <typename RowT, bool NIB>
__global__ __launch_bounds__(kSweepThreads) void k_score_sweep(
    const RowT *__restrict__ rowptr, const uint32_t *__restrict__ tup,
    const uint32_t *__restrict__ boff, const uint8_t *__restrict__ Lc,
    const uint8_t *__restrict__ Ln, const long long *__restrict__ S, uint32_t *__restrict__ E,
    uint8_t *__restrict__ prop, int64_t chunk_lo, int64_t chunk_hi, int slice_base, int k, int ncs,
    int col_bits, int pass, long long P, int64_t gather_limit) {
    extern __shared__ uint32_t smem[];
    const int hist_words = (kSliceRows * k + 1) >> 1;
    uint32_t *hist = smem;                 // hist_words
    uint32_t *bo = hist + hist_words;      // ncs + 1
    uint32_t *room = bo + ncs + 1;         // k
    const int tid = threadIdx.x;
    const int64_t v0 = chunk_lo + (int64_t)blockIdx.x * kSliceRows;
    const int64_t left = chunk_hi - v0;
    const int nv = left < kSliceRows ? (int)left : kSliceRows;
    const int64_t e0 = (int64_t)rowptr[v0];
    const uint32_t *gbo = boff + (size_t)(slice_base + blockIdx.x) * (ncs + 1);

    for (int q = tid; q < hist_words; q += kSweepThreads) hist[q] = 0;
    for (int q = tid; q <= ncs; q += kSweepThreads) bo[q] = gbo[q];
    for (int j = tid; j < k; j += kSweepThreads) room[j] = (uint32_t)(P - S[j]);
    __syncthreads();

    const uint32_t *tbase = tup + e0;
    const uint32_t mask = (1u << col_bits) - 1u;
    constexpr int U = 4;
    for (int j = 0; j < ncs; ++j) {
        const int64_t cb = (int64_t)j << col_bits;
        if (cb >= gather_limit) break;
        const uint32_t b1 = bo[j + 1];
        for (uint32_t base = bo[j] + tid; base < b1; base += kSweepThreads * U) {
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
                    atomicAdd(&hist[c >> 1], 1u << (16 * (c & 1u)));
                }
            }
        }
    }
    __syncthreads();

    // blend and propose, one thread per vertex
    const int sh = pass > 0 ? pass - 1 : 0;
    for (int t = tid; t < nv; t += kSweepThreads) {
        const int64_t v = v0 + t;
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

}  // namespace grem
