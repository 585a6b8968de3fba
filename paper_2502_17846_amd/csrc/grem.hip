// Host side of the GREM library: argument checks, workspace carve-up, and the stream-ordered
// sequence of launches for each chunk of each pass (Alg. 1's chunk loop).  See include/grem.h for
// the contract of every entry point.
#include "grem.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "grem_kernels.hip.h"
#include "grem_twophase.hip.h"

namespace {

using namespace grem;

constexpr int kLdsHistBytes = 32 * 1024;   // LDS spent on one tile's histograms
constexpr int kLdsMaxK = 1024;             // above this the histograms live in E's rows
constexpr int kLongRowDegree = 16384;      // plain score kernels: rows this long get a grid of their own ...
constexpr uint32_t kLongRowPart = 16384;   // ... that many entries per workgroup and turn
constexpr unsigned kLongRowGrid = 512;
constexpr int kSweepMaxK = 16;             // two-phase path: 4-bit labels, 16-bit counters, 2048 rows, 64 KB
constexpr int64_t kSweepMinN = 1 << 22;    // AUTO: label table must exceed L2 for the path to pay
constexpr int64_t kSweepMinChunk = 1 << 14;   // AUTO: per-chunk launches must have work to do
constexpr int kDefaultColBits = 17;        // 2^17 labels, two per byte: 64 KB of LDS, two workgroups per CU
constexpr int64_t kMaxSegments = 1ll << 22;   // chunks * column blocks

struct Global {
    std::mutex mu;
    void *ws = nullptr;
    size_t ws_bytes = 0;
    int hist_mode = GREM_HIST_AUTO;
    int long_row_degree = kLongRowDegree;
    int sweep_col_bits = 0;                // 0 = automatic
    int sweep_hub_degree = 2048;
    bool prof = false;
    struct Ev { int cls; hipEvent_t a, b; };
    std::vector<Ev> events;
    std::vector<hipEvent_t> pool;
};
Global g;

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// Geometry of the two-phase path: chunks, row slices and column blocks (see grem_twophase.hip.h).
struct TpGeom {
    int cb = 0, nbc = 0, nblk = 0, nch = 0, nsl = 0, shift = -1, gb = 0, ngroups = 1;
    uint32_t chunk = 0;
    bool ok = false;
};

TpGeom tp_geometry(int64_t n, int64_t chunk, int col_bits_setting) {
    TpGeom t;
    const int64_t cl = chunk < n ? chunk : n;
    const int64_t nch = (n + cl - 1) / cl;
    const int64_t nsl = (cl + kSliceRows - 1) / kSliceRows;
    int cb = col_bits_setting;
    if (cb == 0) {
        cb = 4;
        while (cb < kDefaultColBits && (1ll << cb) < cl) ++cb;
    }
    const int64_t nbc = (cl + (1ll << cb) - 1) >> cb;
    const int64_t nblk = nch * nbc;
    t.cb = cb;
    t.chunk = (uint32_t)cl;
    for (int b = 0; b < 31; ++b)
        if ((1ll << b) == cl) t.shift = b;
    t.ok = nblk <= kMaxBlocks && nch * nblk <= kMaxSegments && nch * nsl < (1ll << 28) &&
           nch * (nsl + 1) * nblk < (1ll << 40);
    if (t.ok) {
        t.nbc = (int)nbc; t.nblk = (int)nblk; t.nch = (int)nch; t.nsl = (int)nsl;
        // the intermediate copy keeps row (11 bits), block in group (gb) and column in block (cb) in 32 bits
        while (t.gb < 21 - cb && (1ll << t.gb) < nblk) ++t.gb;
        t.ngroups = (int)((nblk + (1ll << t.gb) - 1) >> t.gb);
    }
    return t;
}

struct Layout {
    size_t E, Lc, prop, S, cnt, tot, room, ocnt, fillRank, fillSorted, fillC, misc, long_cnt, long_list;
    // plan of the two-phase path (k <= 16 only)
    size_t sl_reg_cnt, sl_reg_start, sl_nh, sl_hub_start, sl_hent, sl_hent_start, share_h0, share_nhs,
        ch_regtot, ch_nh, ch_H, ch_nvs, ch_hbase, hub_row, hub_off;
    size_t total;
    size_t subR, subH, xstart, tstart, lo, loh, Hhub, T, R, Lx, Rdyn, U, Uh, E16, total_sweep;   // extras of the two-phase path, after `total`
    size_t hub_rows_cap;                                          // rows of Hhub
};

inline int64_t slices_per_chunk(int64_t n, int64_t chunk) {
    const int64_t cl = chunk < n ? chunk : n;
    return (cl + kSliceRows - 1) / kSliceRows;
}

constexpr int kMaxParts = 8;      // parts of a slice (hub share) in the re-layout

Layout make_layout(int64_t n, int64_t nnz, int64_t hub_entries, int32_t k, int64_t chunk, bool external_E,
                   const TpGeom &tp, int hub_degree, bool seeded, int npr = kMaxParts, int nps = kMaxParts) {
    Layout L{};
    const int64_t cl = chunk < n ? chunk : n;
    const size_t lab = k <= 255 ? 1 : 2;
    const int64_t ntiles = (cl + kAdmitTile - 1) / kAdmitTile;
    const int64_t nchunks = (n + chunk - 1) / chunk;
    const size_t G = (size_t)nchunks * (size_t)slices_per_chunk(n, chunk);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
    L.E = take(external_E ? 0 : (size_t)n * (size_t)k * 4);
    L.Lc = take((size_t)n * lab);
    L.prop = take((size_t)cl * lab);
    L.S = take((size_t)k * 8);
    L.cnt = take((size_t)ntiles * (size_t)k * 4);
    L.tot = take(2 * (size_t)k * 4);
    L.room = take((size_t)k * 8);
    L.ocnt = take((size_t)ntiles * 4);
    L.fillRank = take((size_t)k * 4);
    L.fillSorted = take((size_t)k * 8);
    L.fillC = take(((size_t)k + 1) * 8);
    L.misc = take(16 * 8);
    L.long_cnt = take((size_t)nchunks * 4);
    L.long_list = take((size_t)cl * 4);
    const bool tp_possible = k <= kSweepMaxK && tp.ok;
    if (tp_possible) {
        L.sl_reg_cnt = take(G * 4);
        L.sl_reg_start = take(G * 8);
        L.sl_nh = take(G * 4);
        L.sl_hub_start = take(G * 4);
        L.sl_hent = take(G * 8);
        L.sl_hent_start = take(G * 8);
        L.share_h0 = take(G * 4);
        L.share_nhs = take(G * 4);
        L.ch_regtot = take((size_t)nchunks * 8);
        L.ch_nh = take((size_t)nchunks * 4);
        L.ch_H = take((size_t)nchunks * 8);
        L.ch_nvs = take((size_t)nchunks * 4);
        L.ch_hbase = take(((size_t)nchunks + 1) * 8);
        L.hub_row = take((size_t)n * 4);
        L.hub_off = take((size_t)(n + nchunks) * 8);
    }
    L.total = off;
    if (tp_possible) {
        // a chunk cannot hold more hubs than rows, nor more than entries / hub_degree
        size_t hubs = (size_t)(nnz / (hub_degree > 0 ? hub_degree : 1)) + 1;
        if (hubs > (size_t)cl) hubs = (size_t)cl;
        L.hub_rows_cap = hubs;
        const size_t segs = (size_t)tp.nch * (size_t)tp.nblk;
        const size_t rows = (size_t)tp.nch * ((size_t)tp.nsl + 1);
        L.subR = take(rows * (size_t)tp.nblk * 4);
        L.subH = take(rows * (size_t)tp.nblk * 4);
        L.xstart = take((segs + 1) * 8);
        L.tstart = take((segs + 1) * 8);
        L.lo = take(G * (size_t)npr * ((size_t)tp.ngroups + 1) * 4);
        L.loh = take(G * (size_t)nps * ((size_t)tp.ngroups + 1) * 4);
        L.Hhub = take(hubs * (size_t)k * 4);
        // every sub-segment is padded to a multiple of 4 tuples, every segment to a multiple of 8
        const size_t slots = (size_t)(nnz > 0 ? nnz : 0) + 6 * rows * (size_t)tp.nblk + 8 * segs;
        L.T = take(slots * 3 + 16);                 // column in block, 3 bytes per tuple
        L.R = take(slots * 2 + 16);                 // row field, 2 bytes per tuple
        L.Lx = take(slots / 2 + 16);                // label, 4 bits per tuple
        L.Rdyn = take(seeded ? slots * 2 + 16 : 0); // seeded runs: R with the unassigned neighbours marked
        L.U = take((size_t)(nnz > 0 ? nnz : 0) * 4 + 16);
        L.Uh = take((size_t)(hub_entries > 0 ? hub_entries : 0) * 4 + 16);
        L.E16 = take((size_t)n * (size_t)k * 2);
    }
    L.total_sweep = off;
    return L;
}

bool args_ok(const void *rowptr, const int32_t *colidx, int64_t n, int32_t k, double slack,
             int64_t chunk, int32_t R) {
    if (!rowptr || !colidx) return false;
    if (n < 1 || n > (int64_t)INT32_MAX) return false;
    if (k < 1 || k > GREM_MAX_K) return false;
    if (chunk < 1 || R < 0) return false;
    if (!(slack >= 1.0) || std::isinf(slack)) return false;
    return true;
}

// Launch bracket: optional event pair per launch, error check after it.
struct Launcher {
    hipStream_t stream;
    int err = GREM_OK;
    hipEvent_t get_event() {
        if (!g.pool.empty()) { hipEvent_t e = g.pool.back(); g.pool.pop_back(); return e; }
        hipEvent_t e;
        // timing only: no system-scope fence (and the cache write-back it implies) when the event completes
        if (hipEventCreateWithFlags(&e, hipEventDisableSystemFence) != hipSuccess) { err = GREM_ERR_HIP; return nullptr; }
        return e;
    }
    template <typename F> void run(int cls, F &&f) {
        if (err) return;
        hipEvent_t a = nullptr, b = nullptr;
        if (g.prof) {
            a = get_event(); b = get_event();
            if (err) return;
            if (hipEventRecord(a, stream) != hipSuccess) { err = GREM_ERR_HIP; return; }
        }
        f();
        if (hipGetLastError() != hipSuccess) { err = GREM_ERR_HIP; return; }
        if (g.prof) {
            if (hipEventRecord(b, stream) != hipSuccess) { err = GREM_ERR_HIP; return; }
            g.events.push_back({cls, a, b});
        }
    }
};

template <typename RowT, typename LabelT>
int run_partition(const RowT *rowptr, const int32_t *colidx, int64_t n, int32_t k, double slack,
                  int64_t chunk, int32_t R, const int32_t *seed, int32_t *labels_out,
                  int64_t *sizes_out, uint32_t *estimates_out, hipStream_t stream) {
    const long long P = grem_capacity(n, k, slack);
    const bool external_E = estimates_out != nullptr;
    const int hub_degree = g.sweep_hub_degree;
    const TpGeom geo = tp_geometry(n, chunk, g.sweep_col_bits);
    Layout lay = make_layout(n, 0, 0, k, chunk, external_E, geo, hub_degree, seed != nullptr);

    const int hist_mode = g.hist_mode;
    if (hist_mode == GREM_HIST_LDS && k > kLdsMaxK) return GREM_ERR_ARG;
    if (hist_mode == GREM_HIST_SWEEP && (k > kSweepMaxK || !geo.ok)) return GREM_ERR_ARG;
    const bool use_lds = hist_mode != GREM_HIST_GLOBAL && k <= kLdsMaxK;

    // workspace
    char *ws = nullptr, *ws2 = nullptr;
    bool own_ws = false;
    if (g.ws) {
        if (g.ws_bytes < lay.total) return GREM_ERR_NOMEM;
        ws = (char *)g.ws;
    } else {
        if (hipMallocAsync((void **)&ws, lay.total, stream) != hipSuccess) {
            (void)hipGetLastError();
            return GREM_ERR_NOMEM;
        }
        own_ws = true;
    }
    auto release = [&]() {
        if (own_ws) (void)hipFreeAsync(ws, stream);
        if (ws2) (void)hipFreeAsync(ws2, stream);
    };

    uint32_t *E = external_E ? estimates_out : (uint32_t *)(ws + lay.E);
    LabelT *Lc = (LabelT *)(ws + lay.Lc);
    LabelT *prop = (LabelT *)(ws + lay.prop);
    long long *S = (long long *)(ws + lay.S);
    uint32_t *cnt = (uint32_t *)(ws + lay.cnt);
    uint32_t *tot = (uint32_t *)(ws + lay.tot);      // two-phase path: upper bounds of the chunk's movers per partition
    long long *room = (long long *)(ws + lay.room);
    uint32_t *ocnt = (uint32_t *)(ws + lay.ocnt);
    int32_t *fillRank = (int32_t *)(ws + lay.fillRank);
    long long *fillSorted = (long long *)(ws + lay.fillSorted);
    long long *fillC = (long long *)(ws + lay.fillC);
    unsigned long long *misc = (unsigned long long *)(ws + lay.misc);
    uint32_t *long_cnt = (uint32_t *)(ws + lay.long_cnt);
    uint32_t *long_list = (uint32_t *)(ws + lay.long_list);

    Launcher L{stream};

    // ---- prepass + the one validation read-back
    if (hipMemsetAsync(S, 0, (size_t)k * 8, stream) != hipSuccess ||
        hipMemsetAsync(misc, 0, 16 * 8, stream) != hipSuccess) { release(); return GREM_ERR_HIP; }
    {
        int64_t blocks = (n + 255) / 256;
        if (blocks > 256 * 32) blocks = 256 * 32;
        L.run(GREM_KERNEL_PREPASS, [&] {
            hipLaunchKernelGGL((k_prepass<RowT, LabelT>), dim3((unsigned)blocks), dim3(256), 0, stream,
                               rowptr, seed, n, (int)k, Lc, (unsigned long long *)S, misc);
        });
        L.run(GREM_KERNEL_PREPASS, [&] {
            hipLaunchKernelGGL(k_check_seed_sizes, dim3((k + 255) / 256), dim3(256), 0, stream, S, (int)k,
                               P, misc);
        });
    }
    // plan of the two-phase path (needs only rowptr, so it runs before the read-back)
    const int64_t nchunks = (n + chunk - 1) / chunk;
    const int nsl = (int)slices_per_chunk(n, chunk);
    bool sweep = false;
    SweepPlan pl{};
    if constexpr (sizeof(LabelT) == 1) {
        const bool can = k <= kSweepMaxK && geo.ok && (((uintptr_t)E) & 15u) == 0;
        if (hist_mode == GREM_HIST_SWEEP && !can) { release(); return GREM_ERR_ARG; }
        sweep = can && (hist_mode == GREM_HIST_SWEEP ||
                        (hist_mode == GREM_HIST_AUTO && n >= kSweepMinN && (int64_t)geo.chunk >= kSweepMinChunk));
        if (sweep) {
            pl.sl_reg_cnt = (uint32_t *)(ws + lay.sl_reg_cnt);
            pl.sl_reg_start = (u64 *)(ws + lay.sl_reg_start);
            pl.sl_nh = (uint32_t *)(ws + lay.sl_nh);
            pl.sl_hub_start = (uint32_t *)(ws + lay.sl_hub_start);
            pl.sl_hent = (u64 *)(ws + lay.sl_hent);
            pl.sl_hent_start = (u64 *)(ws + lay.sl_hent_start);
            pl.share_h0 = (uint32_t *)(ws + lay.share_h0);
            pl.share_nhs = (uint32_t *)(ws + lay.share_nhs);
            pl.ch_regtot = (u64 *)(ws + lay.ch_regtot);
            pl.ch_nh = (uint32_t *)(ws + lay.ch_nh);
            pl.ch_H = (u64 *)(ws + lay.ch_H);
            pl.ch_nvs = (uint32_t *)(ws + lay.ch_nvs);
            pl.ch_hbase = (u64 *)(ws + lay.ch_hbase);
            pl.hub_row = (int32_t *)(ws + lay.hub_row);
            pl.hub_off = (u64 *)(ws + lay.hub_off);
            const unsigned G = (unsigned)(nchunks * nsl);
            const int64_t cl = (int64_t)geo.chunk;
            L.run(GREM_KERNEL_RELAYOUT, [&] {
                hipLaunchKernelGGL((k_plan_slices<RowT>), dim3(G), dim3(256), 0, stream, rowptr, n, cl, nsl,
                                   (uint32_t)hub_degree, pl);
            });
            L.run(GREM_KERNEL_RELAYOUT, [&] {
                hipLaunchKernelGGL(k_plan_chunks, dim3((unsigned)nchunks), dim3(256), 0, stream, n, cl, nsl,
                                   geo.nblk, pl, misc);
            });
            {
                TpTables only_nch{};
                only_nch.nch = geo.nch;
                L.run(GREM_KERNEL_RELAYOUT, [&] {
                    hipLaunchKernelGGL(k_tp_scan_segments, dim3(1), dim3(1024), 0, stream, only_nch, pl.ch_hbase, 2);
                });
            }

            L.run(GREM_KERNEL_RELAYOUT, [&] {
                hipLaunchKernelGGL((k_plan_hubs<RowT>), dim3(G), dim3(256), 0, stream, rowptr, n, cl, nsl,
                                   (uint32_t)hub_degree, pl);
            });
            L.run(GREM_KERNEL_RELAYOUT, [&] {
                hipLaunchKernelGGL(k_plan_shares, dim3((G + 255) / 256), dim3(256), 0, stream, n, cl, nsl,
                                   (int)G, pl, misc);
            });
        }
    } else {
        if (hist_mode == GREM_HIST_SWEEP) { release(); return GREM_ERR_ARG; }
    }
    if (L.err) { release(); return L.err; }
    unsigned long long h_misc[16] = {0};
    if (hipMemcpyAsync(h_misc, misc, sizeof(h_misc), hipMemcpyDeviceToHost, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess) { release(); return GREM_ERR_HIP; }
    if (h_misc[1] != 0 || h_misc[2] != 0) { release(); return GREM_ERR_SEED; }
    const unsigned long long maxdeg = h_misc[0];
    const int64_t nnz = (int64_t)h_misc[3];
    if (R >= 32 || (maxdeg << R) >= (1ull << 32)) { release(); return GREM_ERR_RANGE; }

    // tile shape of the plain score kernels
    int tv = kGlobalTile;
    if (use_lds) {
        tv = 256;
        while (tv > 1 && (size_t)tv * k * 4 > (size_t)kLdsHistBytes) tv >>= 1;
    }
    if (maxdeg * (unsigned long long)tv >= (1ull << 31)) { release(); return GREM_ERR_RANGE; }
    const size_t score_lds = use_lds ? ((size_t)tv * k + tv + 1 + k) * 4 : ((size_t)tv + 1 + k) * 4;
    const size_t count_lds = (size_t)k * 4;
    const size_t apply_lds = ((size_t)k + (size_t)(kAdmitThreads / 64) * k + 2 * (size_t)k) * 4;
    const size_t fill_lds = (size_t)k * 4;

    if (apply_lds > 64 * 1024 &&
        (hipFuncSetAttribute((const void *)k_apply<LabelT, false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)apply_lds) != hipSuccess ||
         hipFuncSetAttribute((const void *)k_apply<LabelT, true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)apply_lds) != hipSuccess)) { release(); return GREM_ERR_HIP; }

    // ---- two-phase path: allocate its extras, re-lay-out the entries once
    TpTables tb{};
    uint32_t *T = nullptr, *Hhub = nullptr;
    uint16_t *Rw = nullptr, *Rdyn = nullptr, *E16 = nullptr;      // Rw: the tuples' row fields
    uint32_t *Lx = nullptr;
    // estimates of the regular rows of the two-phase path stay below hub_degree * 2^R: 16 bits when that fits
    const bool use16 = (((unsigned long long)(hub_degree - 1)) << R) <= 65535ull;
    size_t tp_score_lds = 0, tp_lookup_lds = 0;
    const int share_hubs = (int)h_misc[5];
    const size_t max_chunk_hubs = (size_t)h_misc[6];
    int lookup_target = 256;                 // workgroups of one look-up launch
    if constexpr (sizeof(LabelT) == 1) {
        auto set_lds = [&](const void *f, size_t bytes) {
            return bytes <= 64 * 1024 ||
                   hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) == hipSuccess;
        };
        if (sweep) {
            lay = make_layout(n, nnz, (int64_t)h_misc[8], k, chunk, external_E, geo, hub_degree, seed != nullptr);
            // (dynamic part: the 64 KB of counters are a static array of the kernel)
            tp_score_lds = ((size_t)kSliceRows / 2 + (size_t)share_hubs * k + 3 * (size_t)k) * 4;
            tp_lookup_lds = (size_t)1 << (geo.cb > 5 ? geo.cb - 1 : 4);
            // a score workgroup must fit the 160 KB of LDS (two per CU do when a share touches few hubs);
            // one share may touch kMaxShareHubs hubs; sub-segment offsets are 32-bit
            const bool fits = tp_score_lds + (size_t)kSliceRows * 32 <= 150 * 1024 && share_hubs <= kMaxShareHubs &&
                              max_chunk_hubs <= lay.hub_rows_cap &&
                              h_misc[7] + 8ull * ((unsigned long long)geo.nsl + 2) * geo.nblk < (1ull << 32);
            if (!fits) {
                if (hist_mode == GREM_HIST_SWEEP) { release(); return GREM_ERR_ARG; }
                sweep = false;
            }
        }
        if (sweep) {
            char *xbase = nullptr;
            if (g.ws) {
                if (g.ws_bytes >= lay.total_sweep) xbase = ws;
                else if (hist_mode == GREM_HIST_SWEEP) { release(); return GREM_ERR_NOMEM; }
                else sweep = false;
            } else {
                if (hipMallocAsync((void **)&ws2, lay.total_sweep - lay.total, stream) != hipSuccess) {
                    (void)hipGetLastError();
                    ws2 = nullptr;
                    if (hist_mode == GREM_HIST_SWEEP) { release(); return GREM_ERR_NOMEM; }
                    sweep = false;
                } else {
                    xbase = ws2 - lay.total;
                }
            }
            if (sweep) {
                tb.subR = (uint32_t *)(xbase + lay.subR);
                tb.subH = (uint32_t *)(xbase + lay.subH);
                tb.xstart = (u64 *)(xbase + lay.xstart);
                tb.tstart = (u64 *)(xbase + lay.tstart);
                tb.chunk = geo.chunk;
                tb.chunk_shift = geo.shift;
                {   // round-up magic number: exact for dividends below 2^31 (vertex ids are)
                    uint32_t sh = 0;
                    while ((1ull << sh) < geo.chunk) ++sh;
                    tb.chunk_magic_shift = sh > 0 ? sh - 1 : 0;
                    tb.chunk_magic = geo.chunk > 1
                        ? (uint32_t)((((unsigned long long)1 << (32 + tb.chunk_magic_shift)) + geo.chunk - 1) / geo.chunk)
                        : 0u;
                    if (geo.chunk == 1) tb.chunk_shift = 0;
                }
                tb.nch = geo.nch;
                tb.nsl = geo.nsl;
                tb.nbc = geo.nbc;
                tb.nblk = geo.nblk;
                tb.cb = geo.cb;
                Hhub = (uint32_t *)(xbase + lay.Hhub);
                T = (uint32_t *)(xbase + lay.T);
                Rw = (uint16_t *)(xbase + lay.R);
                Lx = (uint32_t *)(xbase + lay.Lx);
                Rdyn = seed ? (uint16_t *)(xbase + lay.Rdyn) : nullptr;
                E16 = (uint16_t *)(xbase + lay.E16);
                tb.gb = geo.gb;
                tb.ngroups = geo.ngroups;
                tb.lo = (uint32_t *)(xbase + lay.lo);
                tb.loh = (uint32_t *)(xbase + lay.loh);
                uint32_t *U = (uint32_t *)(xbase + lay.U);
                uint32_t *Uh = (uint32_t *)(xbase + lay.Uh);
                // step 1 collects a unit's tuples in LDS: cut the slices (shares) in as many parts as it
                // takes for the largest to fit, two workgroups per CU
                constexpr size_t kGroupLds = 79 * 1024, kPlaceLds = 52 * 1024;
                auto group_fixed = [&](bool share, int np) {
                    return (tp_source_words(share, np, share_hubs) + (size_t)geo.nblk + (size_t)geo.ngroups + 1 + kTpThreads / 64) * 4;
                };
                auto group_cap = [&](bool share, int np) {
                    const size_t fixed = group_fixed(share, np);
                    return (uint32_t)(kGroupLds > fixed ? (kGroupLds - fixed) / 4 : 0);
                };
                int npr = 1, nps = 1;
                // ... and, if that takes no more than kMaxParts, so small that a thread holds its share of the
                // unit's entries in registers (one round of kTpThreads * kTpBatch entries)
                const unsigned long long one_round = (unsigned long long)kTpThreads * kTpBatch;
                auto fits = [&](bool share, int np, unsigned long long most, bool in_regs) {
                    const unsigned long long unit = most / np + most / (8ull * np) + 64;
                    return group_cap(share, np) >= unit && (!in_regs || unit <= one_round);
                };
                while (npr < kMaxParts && !fits(false, npr, h_misc[9], false)) npr *= 2;
                while (nps < kMaxParts && !fits(true, nps, h_misc[10], false)) nps += 1;
                {
                    // slices differ in size: it is the average one whose parts should take one round (the
                    // larger ones take two, and their tuples still fit LDS)
                    const unsigned long long avg_slice =
                        ((unsigned long long)nnz - h_misc[8]) / (unsigned long long)(nchunks * nsl) + 1;
                    int a = npr, b = nps;
                    while (a < kMaxParts && !fits(false, a, avg_slice, true)) a *= 2;
                    while (b < kMaxParts && !fits(true, b, h_misc[10], true)) b += 1;
                    if (fits(false, a, avg_slice, true) && fits(false, a, h_misc[9], false)) npr = a;
                    if (fits(true, b, h_misc[10], true)) nps = b;
                }
                tb.npr = npr;
                tb.nps = nps;
                const uint32_t capR = group_cap(false, npr), capS = group_cap(true, nps);
                const size_t groupR_lds = group_fixed(false, npr) + (size_t)capR * 4;
                const size_t groupS_lds = group_fixed(true, nps) + (size_t)capS * 4;
                // step 2: up to 8 slices at a time
                const int nbg = geo.nblk < (1 << geo.gb) ? geo.nblk : (1 << geo.gb);
                int batch = 8192 / nbg;
                if (batch > 8) batch = 8;
                if (batch < 1) batch = 1;
                const int maxruns = batch * (npr > nps ? npr : nps);
                const size_t place_fixed = (2 * (size_t)nbg + maxruns) * 8 +
                                           ((size_t)2 * maxruns + 1 + 2 * (size_t)nbg + 1 + (size_t)batch * nbg) * 4;
                const uint32_t capP = (uint32_t)(kPlaceLds > place_fixed ? (kPlaceLds - place_fixed) / 4 : 0);
                const size_t place_lds = place_fixed + (size_t)capP * 4;
                const size_t rows = (size_t)geo.nch * ((size_t)geo.nsl + 1);
                if (hipMemsetAsync(Hhub, 0, lay.hub_rows_cap * (size_t)k * 4, stream) != hipSuccess ||
                    hipMemsetAsync(tb.subR, 0, rows * (size_t)geo.nblk * 4, stream) != hipSuccess ||
                    hipMemsetAsync(tb.subH, 0, rows * (size_t)geo.nblk * 4, stream) != hipSuccess ||
                    !set_lds((const void *)k_tp_group<RowT, false>, groupR_lds) ||
                    !set_lds((const void *)k_tp_group<RowT, true>, groupS_lds) ||
                    !set_lds((const void *)k_tp_place<RowT>, place_lds) ||
                    !set_lds((const void *)k_tp_lookup<true, false>, tp_lookup_lds) ||
                    !set_lds((const void *)k_tp_lookup<true, true>, tp_lookup_lds) ||
                    !set_lds((const void *)k_tp_score<RowT, uint32_t>, tp_score_lds) ||
                    !set_lds((const void *)k_tp_score<RowT, uint16_t>, tp_score_lds)) {
                    release();
                    return GREM_ERR_HIP;
                }
                lookup_target = tp_lookup_lds > 80 * 1024 ? 256 : 512;
                const unsigned G = (unsigned)(nchunks * nsl);
                const unsigned segs = (unsigned)((int64_t)geo.nch * geo.nblk);
                L.run(GREM_KERNEL_RELAYOUT, [&] {
                    hipLaunchKernelGGL((k_tp_group<RowT, false>), dim3(G * (unsigned)npr), dim3(kTpThreads),
                                       groupR_lds, stream, rowptr, colidx, n, (uint32_t)hub_degree, pl, tb,
                                       share_hubs, capR, (int)nsl, U);
                });
                // shares: no chunk has more than max_shares of them (none at all: nothing to launch)
                const unsigned max_shares = (unsigned)h_misc[11];
                if (max_shares != 0)
                    L.run(GREM_KERNEL_RELAYOUT, [&] {
                        hipLaunchKernelGGL((k_tp_group<RowT, true>),
                                           dim3((unsigned)nchunks * max_shares * (unsigned)nps), dim3(kTpThreads),
                                           groupS_lds, stream, rowptr, colidx, n, (uint32_t)hub_degree, pl, tb,
                                           share_hubs, capS, (int)max_shares, Uh);
                    });
                L.run(GREM_KERNEL_RELAYOUT, [&] {
                    hipLaunchKernelGGL(k_tp_scan_slices, dim3((segs + 255) / 256), dim3(256), 0, stream, tb);
                });
                L.run(GREM_KERNEL_RELAYOUT, [&] {
                    hipLaunchKernelGGL(k_tp_scan_segments, dim3(2), dim3(1024), 0, stream, tb, pl.ch_hbase, 0);
                });
                L.run(GREM_KERNEL_RELAYOUT, [&] {
                    hipLaunchKernelGGL((k_tp_place<RowT>), dim3((unsigned)((int64_t)geo.ngroups * geo.nch)),
                                       dim3(kPlaceThreads), place_lds, stream, rowptr, n, pl, tb, U, Uh, T, Rw, batch,
                                       capP);
                });
            }
        }
    }

    // look-ups of the labels of chunks [c0, c0 + count): shares per column block sized so that one
    // launch fills the chip without cutting the blocks' streams into crumbs
    // `mark`: seeded runs, first pass: the row fields the score kernels read are those of Rdyn, where
    // bit 15 also marks the tuples whose neighbour is unassigned (set by the initial look-up from global
    // memory, cleared by the look-up of the neighbour's chunk)
    auto lookup = [&](int c0, int count, int cmin, bool from_lds, bool mark) {
        if constexpr (sizeof(LabelT) == 1) {
            if (cmin >= geo.nch) return;
            const int64_t per_block = nnz / geo.nblk + 1;
            int spb = lookup_target / geo.nbc;
            const int64_t by_work = per_block / 8192 + 1;
            if (spb > by_work) spb = (int)by_work;
            if (spb < 1) spb = 1;
            const dim3 grid((unsigned)(geo.nbc * spb), (unsigned)count);
            L.run(GREM_KERNEL_LOOKUP, [&] {
                if (!from_lds)
                    hipLaunchKernelGGL((k_tp_lookup<false, true>), grid, dim3(kTpThreads), 0, stream, T, Lx, Rw, Rdyn,
                                       tb, (const uint8_t *)Lc, n, c0, cmin, spb);
                else if (mark)
                    hipLaunchKernelGGL((k_tp_lookup<true, true>), grid, dim3(kTpThreads), tp_lookup_lds, stream, T,
                                       Lx, Rw, Rdyn, tb, (const uint8_t *)Lc, n, c0, cmin, spb);
                else
                    hipLaunchKernelGGL((k_tp_lookup<true, false>), grid, dim3(kTpThreads), tp_lookup_lds, stream, T,
                                       Lx, Rw, Rdyn, tb, (const uint8_t *)Lc, n, c0, cmin, spb);
            });
        }
    };
    if (sweep && seed) {        // the seeds are the labels every first-pass look-up starts from
        for (int c0 = 0; c0 < geo.nch; c0 += 32768) {
            const int count = geo.nch - c0 < 32768 ? geo.nch - c0 : 32768;
            lookup(c0, count, 0, false, true);
        }
    }

    // plain score kernels: rows this long are taken out of their tile and spread over a grid of their own
    const bool split_long = !sweep && maxdeg >= (unsigned long long)g.long_row_degree;
    const size_t long_lds = (size_t)k * 4;
    if (split_long && long_lds > 64 * 1024 &&
        hipFuncSetAttribute((const void *)k_long_rows<RowT, LabelT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)long_lds) != hipSuccess) { release(); return GREM_ERR_HIP; }

    for (int pass = 0; pass <= R && !L.err; ++pass) {
        if (split_long && hipMemsetAsync(long_cnt, 0, (size_t)nchunks * 4, stream) != hipSuccess) {
            release();
            return GREM_ERR_HIP;
        }
        for (int64_t c = 0; c < nchunks && !L.err; ++c) {
            const int64_t lo = c * chunk;
            const int64_t hi = (lo + chunk < n) ? lo + chunk : n;
            const int64_t len = hi - lo;
            const int64_t gather_limit = (pass == 0 && !seed) ? lo : n;
            const unsigned admit_blocks = (unsigned)((len + kAdmitTile - 1) / kAdmitTile);
            if (sweep) {
                if constexpr (sizeof(LabelT) == 1) {
                    const unsigned blocks = (unsigned)((len + kSliceRows - 1) / kSliceRows);
                    const int jlim = (pass == 0 && !seed) ? (int)c * geo.nbc : geo.nblk;
                    // the estimates are state between passes and, if the caller asked for them, output:
                    // the last pass does not store them otherwise
                    const int store_e = (pass < R || external_E) ? 1 : 0;
                    const uint16_t *rows_now = (seed && pass == 0) ? Rdyn : Rw;
                    L.run(GREM_KERNEL_SCORE, [&] {
                        if (use16)
                            hipLaunchKernelGGL((k_tp_score<RowT, uint16_t>), dim3(blocks), dim3(kTpThreads),
                                               tp_score_lds, stream, rowptr, rows_now, Lx, tb, pl, (const uint8_t *)Lc, S, E16,
                                               Hhub, (uint8_t *)prop, cnt, room, (int)c, lo, hi, (int)k, jlim,
                                               share_hubs, (uint32_t)hub_degree, pass, P, store_e);
                        else
                            hipLaunchKernelGGL((k_tp_score<RowT, uint32_t>), dim3(blocks), dim3(kTpThreads),
                                               tp_score_lds, stream, rowptr, rows_now, Lx, tb, pl, (const uint8_t *)Lc, S, E,
                                               Hhub, (uint8_t *)prop, cnt, room, (int)c, lo, hi, (int)k, jlim,
                                               share_hubs, (uint32_t)hub_degree, pass, P, store_e);
                    });
                    // (one workgroup more than the hubs need: it adds up the chunk's mover counts)
                    L.run(GREM_KERNEL_HUBS, [&] {
                        hipLaunchKernelGGL(k_hub_finalize, dim3((unsigned)((max_chunk_hubs + 15) / 16) + 1),
                                           dim3(256), 0, stream, pl, (const uint8_t *)Lc, room, E, Hhub,
                                           (uint8_t *)prop, cnt, (int)c, lo, (int)k, pass, store_e,
                                           (int)admit_blocks, tot);
                    });
                }
            } else {
                const LongRows lr{split_long ? (uint32_t)g.long_row_degree : 0xFFFFFFFFu, kLongRowPart,
                                  long_cnt + c, long_list};
                const unsigned score_blocks = (unsigned)((len + tv - 1) / tv);
                L.run(GREM_KERNEL_SCORE, [&] {
                    if (use_lds)
                        hipLaunchKernelGGL((k_score_lds<RowT, LabelT>), dim3(score_blocks),
                                           dim3(kScoreThreads), score_lds, stream, rowptr, colidx, Lc, S, E,
                                           prop, lo, hi, (int)k, tv, pass, P, gather_limit, lr);
                    else
                        hipLaunchKernelGGL((k_score_global<RowT, LabelT>), dim3(score_blocks),
                                           dim3(kScoreThreads), score_lds, stream, rowptr, colidx, Lc, S, E,
                                           prop, lo, hi, (int)k, pass, P, gather_limit, lr);
                });
                if (split_long) {
                    L.run(GREM_KERNEL_HUBS, [&] {
                        hipLaunchKernelGGL((k_long_rows<RowT, LabelT>), dim3(kLongRowGrid), dim3(kScoreThreads),
                                           long_lds, stream, rowptr, colidx, Lc, E, (int)k, pass, gather_limit, lr);
                    });
                    L.run(GREM_KERNEL_HUBS, [&] {
                        hipLaunchKernelGGL((k_long_propose<LabelT>), dim3(64), dim3(64), 0, stream, Lc, S, E, prop,
                                           lo, (int)k, pass, P, lr);
                    });
                }
            }
            // admission: per-tile mover counts, their prefix over the tiles, ranks.  The two-phase score
            // kernel has already counted the movers and taken the sizes' snapshot, and its tiles are few
            // enough per partition that every k_apply workgroup adds up the earlier tiles' counts itself.
            if (!sweep) {
                L.run(GREM_KERNEL_COUNT, [&] {
                    hipLaunchKernelGGL((k_count<LabelT>), dim3(admit_blocks), dim3(kAdmitThreads), count_lds,
                                       stream, Lc, prop, lo, hi, (int)k, cnt);
                });
                L.run(GREM_KERNEL_SCAN, [&] {
                    hipLaunchKernelGGL(k_scan, dim3(1), dim3(kScanThreads), 0, stream, cnt, (int)admit_blocks,
                                       (int)k, S, P, room);
                });
                L.run(GREM_KERNEL_APPLY, [&] {
                    hipLaunchKernelGGL((k_apply<LabelT, false>), dim3(admit_blocks), dim3(kAdmitThreads),
                                       apply_lds, stream, Lc, prop, lo, hi, (int)k, cnt, room,
                                       (unsigned long long *)S, ocnt, pass);
                });
            } else {
                if constexpr (sizeof(LabelT) == 1) {
                    L.run(GREM_KERNEL_APPLY, [&] {
                        hipLaunchKernelGGL(k_apply16, dim3((admit_blocks + kApply16Tiles - 1) / kApply16Tiles), dim3(kAdmitTile), 0, stream,
                                           (uint8_t *)Lc, (const uint8_t *)prop, lo, hi, (int)k, cnt, room,
                                           tot, (unsigned long long *)S, ocnt, pass);
                    });
                }
            }
            if (pass == 0) {
                L.run(GREM_KERNEL_SPILL_SCAN, [&] {
                    hipLaunchKernelGGL(k_spill_scan, dim3(1), dim3(kScanThreads), 0, stream, ocnt,
                                       (int)admit_blocks, (int)k, S, fillRank, fillSorted, fillC, misc);
                });
                L.run(GREM_KERNEL_SPILL_FILL, [&] {
                    hipLaunchKernelGGL((k_spill_fill<LabelT>), dim3(admit_blocks), dim3(kAdmitThreads),
                                       fill_lds, stream, Lc, lo, hi, (int)k, ocnt, fillRank, fillC,
                                       (unsigned long long *)S, misc);
                });
            }
            // the chunk's new labels, looked up for every row that will read them: rows of later
            // chunks in this pass, rows of this and earlier chunks in the next pass (if there is one)
            if (sweep) lookup((int)c, 1, pass == R ? (int)c + 1 : 0, true, seed != nullptr && pass == 0);
        }
    }
    {
        int64_t blocks = (n + 255) / 256;
        if (blocks > 256 * 32) blocks = 256 * 32;
        L.run(GREM_KERNEL_EXPAND, [&] {
            hipLaunchKernelGGL((k_expand<LabelT>), dim3((unsigned)blocks), dim3(256), 0, stream, Lc, n,
                               labels_out);
        });
        if constexpr (sizeof(LabelT) == 1) {
            if (sweep && use16 && external_E)
                L.run(GREM_KERNEL_EXPAND, [&] {
                    hipLaunchKernelGGL((k_expand_estimates<RowT>), dim3((unsigned)blocks), dim3(256), 0, stream,
                                       rowptr, n, (int)k, (uint32_t)hub_degree, E16, estimates_out);
                });
        }
        if (sizes_out)
            L.run(GREM_KERNEL_EXPAND, [&] {
                hipLaunchKernelGGL(k_copy_sizes, dim3((k + 255) / 256), dim3(256), 0, stream, S, (int)k,
                                   sizes_out);
            });
    }
    release();
    return L.err;
}

template <typename RowT>
int dispatch_labels(const RowT *rowptr, const int32_t *colidx, int64_t n, int32_t k, double slack,
                    int64_t chunk, int32_t R, const int32_t *seed, int32_t *labels_out,
                    int64_t *sizes_out, uint32_t *estimates_out, void *stream) {
    if (!args_ok(rowptr, colidx, n, k, slack, chunk, R) || !labels_out) return GREM_ERR_ARG;
    std::lock_guard<std::mutex> lock(g.mu);
    hipStream_t s = (hipStream_t)stream;
    if (k <= 255)
        return run_partition<RowT, uint8_t>(rowptr, colidx, n, k, slack, chunk, R, seed, labels_out,
                                            sizes_out, estimates_out, s);
    return run_partition<RowT, uint16_t>(rowptr, colidx, n, k, slack, chunk, R, seed, labels_out,
                                         sizes_out, estimates_out, s);
}

template <typename RowT>
int run_edge_cut(const RowT *rowptr, const int32_t *colidx, int64_t n, const int32_t *labels,
                 int64_t *out, void *stream) {
    if (!rowptr || !colidx || !labels || !out || n < 1 || n > (int64_t)INT32_MAX) return GREM_ERR_ARG;
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(k_zero_u64, dim3(1), dim3(64), 0, s, (unsigned long long *)out, 1);
    const unsigned blocks = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL((k_edge_cut<RowT>), dim3(blocks), dim3(256), 0, s, rowptr, colidx, n, labels,
                       (unsigned long long *)out);
    return hipGetLastError() == hipSuccess ? GREM_OK : GREM_ERR_HIP;
}

}  // namespace

extern "C" {

int64_t grem_capacity(int64_t n, int32_t k, double balance_slack) {
    if (n < 1 || k < 1 || !(balance_slack >= 1.0)) return -1;
    const int64_t even = (n + k - 1) / k;
    const double scaled = (double)n * balance_slack;
    const double per = scaled / (double)k;
    const int64_t widened = (int64_t)std::ceil(per);
    return even > widened ? even : widened;
}

size_t grem_workspace_bytes(int64_t n, int64_t nnz, int32_t k, int64_t chunk) {
    if (n < 1 || nnz < 0 || k < 1 || k > GREM_MAX_K || chunk < 1) return 0;
    std::lock_guard<std::mutex> lock(g.mu);
    const TpGeom geo = tp_geometry(n, chunk, g.sweep_col_bits);
    const Layout lay = make_layout(n, nnz, nnz, k, chunk, false, geo, g.sweep_hub_degree, true);
    return lay.total_sweep;
}

int grem_set_workspace(void *dev_ptr, size_t bytes) {
    std::lock_guard<std::mutex> lock(g.mu);
    if ((dev_ptr == nullptr) != (bytes == 0)) return GREM_ERR_ARG;
    if (((uintptr_t)dev_ptr & 255u) != 0) return GREM_ERR_ARG;
    g.ws = dev_ptr;
    g.ws_bytes = bytes;
    return GREM_OK;
}

int grem_set_histogram_mode(int32_t mode) {
    if (mode != GREM_HIST_AUTO && mode != GREM_HIST_LDS && mode != GREM_HIST_GLOBAL &&
        mode != GREM_HIST_SWEEP)
        return GREM_ERR_ARG;
    std::lock_guard<std::mutex> lock(g.mu);
    g.hist_mode = mode;
    return GREM_OK;
}

int grem_set_sweep_hub_degree(int32_t degree) {
    if (degree < 1 || degree > 65535) return GREM_ERR_ARG;
    std::lock_guard<std::mutex> lock(g.mu);
    g.sweep_hub_degree = degree;
    return GREM_OK;
}

int grem_set_long_row_degree(int32_t degree) {
    if (degree < 0) return GREM_ERR_ARG;
    std::lock_guard<std::mutex> lock(g.mu);
    g.long_row_degree = degree == 0 ? kLongRowDegree : degree;
    return GREM_OK;
}

int grem_set_sweep_col_bits(int32_t bits) {
    if (bits != 0 && (bits < 4 || bits > kMaxColBits)) return GREM_ERR_ARG;
    std::lock_guard<std::mutex> lock(g.mu);
    g.sweep_col_bits = bits;
    return GREM_OK;
}

int grem_partition(const int64_t *rowptr, const int32_t *colidx, int64_t n, int32_t k,
                   double balance_slack, int64_t chunk, int32_t refine_passes, int32_t *labels_out,
                   void *stream) {
    return dispatch_labels<int64_t>(rowptr, colidx, n, k, balance_slack, chunk, refine_passes, nullptr,
                                    labels_out, nullptr, nullptr, stream);
}

int grem_partition_seeded(const int64_t *rowptr, const int32_t *colidx, int64_t n, int32_t k,
                          double balance_slack, int64_t chunk, int32_t refine_passes,
                          const int32_t *seed_labels, int32_t *labels_out, void *stream) {
    return dispatch_labels<int64_t>(rowptr, colidx, n, k, balance_slack, chunk, refine_passes,
                                    seed_labels, labels_out, nullptr, nullptr, stream);
}

int grem_partition_r32(const int32_t *rowptr, const int32_t *colidx, int64_t n, int32_t k,
                       double balance_slack, int64_t chunk, int32_t refine_passes, int32_t *labels_out,
                       void *stream) {
    return dispatch_labels<int32_t>(rowptr, colidx, n, k, balance_slack, chunk, refine_passes, nullptr,
                                    labels_out, nullptr, nullptr, stream);
}

int grem_partition_seeded_r32(const int32_t *rowptr, const int32_t *colidx, int64_t n, int32_t k,
                              double balance_slack, int64_t chunk, int32_t refine_passes,
                              const int32_t *seed_labels, int32_t *labels_out, void *stream) {
    return dispatch_labels<int32_t>(rowptr, colidx, n, k, balance_slack, chunk, refine_passes,
                                    seed_labels, labels_out, nullptr, nullptr, stream);
}

int grem_partition_state(const void *rowptr, int32_t rowptr_bits, const int32_t *colidx, int64_t n,
                         int32_t k, double balance_slack, int64_t chunk, int32_t refine_passes,
                         const int32_t *seed_labels, int32_t *labels_out, int64_t *sizes_out,
                         uint32_t *estimates_out, void *stream) {
    if (rowptr_bits == 64)
        return dispatch_labels<int64_t>((const int64_t *)rowptr, colidx, n, k, balance_slack, chunk,
                                        refine_passes, seed_labels, labels_out, sizes_out,
                                        estimates_out, stream);
    if (rowptr_bits == 32)
        return dispatch_labels<int32_t>((const int32_t *)rowptr, colidx, n, k, balance_slack, chunk,
                                        refine_passes, seed_labels, labels_out, sizes_out,
                                        estimates_out, stream);
    return GREM_ERR_ARG;
}

int grem_edge_cut(const int64_t *rowptr, const int32_t *colidx, int64_t n, const int32_t *labels,
                  int64_t *cut_entries_out, void *stream) {
    return run_edge_cut<int64_t>(rowptr, colidx, n, labels, cut_entries_out, stream);
}

int grem_edge_cut_r32(const int32_t *rowptr, const int32_t *colidx, int64_t n, const int32_t *labels,
                      int64_t *cut_entries_out, void *stream) {
    return run_edge_cut<int32_t>(rowptr, colidx, n, labels, cut_entries_out, stream);
}

int grem_profile_enable(int32_t on) {
    std::lock_guard<std::mutex> lock(g.mu);
    g.prof = on != 0;
    return GREM_OK;
}

int grem_profile_reset(void) {
    std::lock_guard<std::mutex> lock(g.mu);
    for (auto &e : g.events) { g.pool.push_back(e.a); g.pool.push_back(e.b); }
    g.events.clear();
    return GREM_OK;
}

int grem_profile_read(int32_t kernel_class, double *total_ms, int64_t *launches) {
    if (kernel_class < 0 || kernel_class >= GREM_KERNEL_CLASSES || !total_ms || !launches)
        return GREM_ERR_ARG;
    std::lock_guard<std::mutex> lock(g.mu);
    double tot = 0.0;
    int64_t cnt = 0;
    for (auto &e : g.events) {
        if (e.cls != kernel_class) continue;
        if (hipEventSynchronize(e.b) != hipSuccess) return GREM_ERR_HIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, e.a, e.b) != hipSuccess) return GREM_ERR_HIP;
        tot += ms;
        cnt += 1;
    }
    *total_ms = tot;
    *launches = cnt;
    return GREM_OK;
}

const char *grem_status_string(int code) {
    switch (code) {
        case GREM_OK: return "ok";
        case GREM_ERR_ARG: return "bad argument";
        case GREM_ERR_NOMEM: return "workspace allocation failed or workspace too small";
        case GREM_ERR_HIP: return "HIP runtime error";
        case GREM_ERR_RANGE: return "max degree * 2^refine_passes does not fit the estimates";
        case GREM_ERR_SEED: return "invalid seed labels";
        case GREM_ERR_LIMIT: return "input larger than the entry point's fixed-size buffer allows";
        default: return "unknown status";
    }
}

const char *grem_kernel_name(int32_t kernel_class) {
    switch (kernel_class) {
        case GREM_KERNEL_PREPASS: return "prepass";
        case GREM_KERNEL_SCORE: return "score";
        case GREM_KERNEL_COUNT: return "count";
        case GREM_KERNEL_SCAN: return "scan";
        case GREM_KERNEL_APPLY: return "apply";
        case GREM_KERNEL_SPILL_SCAN: return "spill_scan";
        case GREM_KERNEL_SPILL_FILL: return "spill_fill";
        case GREM_KERNEL_EXPAND: return "expand";
        case GREM_KERNEL_RELAYOUT: return "relayout";
        case GREM_KERNEL_LOOKUP: return "lookup";
        case GREM_KERNEL_HUBS: return "hub_finalize";
        default: return "?";
    }
}

}  // extern "C"
