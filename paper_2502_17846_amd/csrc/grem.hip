// Host side of the GREM library: argument checks, memory carve-up, and the stream-ordered sequence
// of launches for each chunk of each pass (Alg. 1's chunk loop).  See include/grem.h for the
// contract of every entry point.
//
// Structure:
//   Arena / carve      device memory for a call: pieces of the caller's workspace, or stream-ordered
//                      allocations
//   PlanData           the re-laid-out copy of a graph's entries for the two-phase route (k <= 32):
//                      built once per call, or once per graph behind a grem_plan
//   run_two_phase      Alg. 1's loop on a plan
//   run_plain          Alg. 1's loop straight on the CSR (any k)
#include "grem.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
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
constexpr int kSweepMaxK = 32;             // two-phase route: 16-bit counters for 2048 rows: 64 KB of LDS up to k = 16
                                           // (4-bit labels), 128 KB up to k = 32 (8-bit labels)
constexpr int kHubsPerShare16 = 1024;      // hubs one hub share may touch: their 32-bit counters share the
constexpr int kHubsPerShare32 = 96;        // workgroup's LDS with the slice's counters
constexpr int64_t kSweepMinN = 1 << 22;    // AUTO: label table must exceed L2 for the route to pay
constexpr int64_t kSweepMinChunk = 1 << 14;   // AUTO: per-chunk launches must have work to do
constexpr int kDefaultColBits = 17;        // 2^17 labels, two per byte: 64 KB of LDS, two workgroups per CU
constexpr int kDefaultColBits32 = 16;      // k > 16: 2^16 labels, a byte each
constexpr int kDefaultHubDegree = 8192;
constexpr int64_t kMaxSegments = 1ll << 22;   // chunks * column blocks
constexpr int kMaxParts = kPlanParts;      // parts of a slice (hub share) in the re-layout

// ---- process-wide state: the optional workspace and the measurement aids --------------------------
struct Global {
    std::mutex mu;
    void *ws = nullptr;
    size_t ws_bytes = 0;
    int prof_level = 0;
    struct Ev { int cls; hipEvent_t a, b; };
    std::vector<Ev> events;            // level 2: a pair per launch
    std::vector<hipEvent_t> marks;     // level 1: call start, first pass, end of every pass, end of call
    std::vector<hipEvent_t> pool;
};
Global g;

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// ---- options ---------------------------------------------------------------------------------------
struct Opts {
    int hist_mode = GREM_HIST_AUTO;
    int col_bits = 0;                       // 0 = automatic
    int hub_degree = kDefaultHubDegree;
    int long_row_degree = kLongRowDegree;
    int plan_max_k = 16;
};

bool resolve_options(const grem_options *o, Opts *out) {
    Opts r;
    if (o) {
        if (o->histogram_mode != GREM_HIST_AUTO && o->histogram_mode != GREM_HIST_LDS &&
            o->histogram_mode != GREM_HIST_GLOBAL && o->histogram_mode != GREM_HIST_SWEEP)
            return false;
        if (o->col_bits != 0 && (o->col_bits < 4 || o->col_bits > kMaxColBits)) return false;
        if (o->hub_degree < 0 || o->hub_degree > 65535) return false;
        if (o->long_row_degree < 0) return false;
        if (o->plan_max_k < 0 || o->plan_max_k > kSweepMaxK) return false;
        for (int i = 0; i < 3; ++i)
            if (o->reserved[i] != 0) return false;
        r.hist_mode = o->histogram_mode;
        r.col_bits = o->col_bits;
        if (o->hub_degree) r.hub_degree = o->hub_degree;
        if (o->long_row_degree) r.long_row_degree = o->long_row_degree;
        if (o->plan_max_k) r.plan_max_k = o->plan_max_k;
    }
    *out = r;
    return true;
}

// ---- device memory of a call -----------------------------------------------------------------------
// Bump mode: pieces of one caller-owned block, released by moving the top back.  Otherwise every
// request is an allocation of its own: stream-ordered (released stream-ordered) or, for memory that
// outlives the call, hipMalloc.
struct Arena {
    char *base = nullptr;
    size_t cap = 0, off = 0;
    hipStream_t stream = nullptr;
    bool persistent = false;
    std::vector<void *> owned;
    size_t total = 0;                       // bytes handed out (allocation modes)

    char *alloc(size_t bytes) {
        bytes = align_up(bytes ? bytes : 1);
        if (base) {
            if (off + bytes > cap) return nullptr;
            char *p = base + off;
            off += bytes;
            return p;
        }
        void *p = nullptr;
        const hipError_t e = persistent ? hipMalloc(&p, bytes) : hipMallocAsync(&p, bytes, stream);
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        owned.push_back(p);
        total += bytes;
        return (char *)p;
    }
    struct Mark { size_t off, count; };
    Mark mark() const { return {off, owned.size()}; }
    // gives back everything handed out since `m` (work already enqueued on the stream may still use it:
    // stream-ordered release, and in bump mode whatever takes the space next runs later on the same stream)
    void release_to(Mark m) {
        off = m.off;
        while (owned.size() > m.count) {
            if (persistent) (void)hipFree(owned.back());
            else (void)hipFreeAsync(owned.back(), stream);
            owned.pop_back();
        }
    }
    void release_all() { release_to({0, 0}); }
};

// Several arrays out of one request: the same function lays them out twice, first against a null
// base to find the size, then against the block.
struct Carver {
    char *base;
    size_t off = 0;
    // (an array of no elements is a null pointer, not the address of whatever comes next: code that asks
    // "is there such an array" must not be told yes)
    template <typename T> void take(T *&p, size_t count) {
        p = (base && count) ? reinterpret_cast<T *>(base + off) : nullptr;
        off += align_up(count * sizeof(T));
    }
};
template <typename F> bool carve(Arena &A, F &&f) {
    Carver dry{nullptr};
    f(dry);
    char *p = A.alloc(dry.off);
    if (!p) return false;
    Carver wet{p};
    f(wet);
    return true;
}
template <typename F> size_t carve_size(F &&f) {
    Carver dry{nullptr};
    f(dry);
    return align_up(dry.off ? dry.off : 1);
}

// ---- geometry of the two-phase route: chunks, row slices and column blocks (grem_twophase.hip.h) ---
struct TpGeom {
    int cb = 0, nbc = 0, nblk = 0, nch = 0, nsl = 0, shift = -1, gb = 0, ngroups = 1;
    uint32_t chunk = 0;
    bool ok = false;
};

// kmax: the largest k the layout is to serve (above 16 the look-up keeps a byte per label in LDS)
TpGeom tp_geometry(int64_t n, int64_t chunk, int col_bits_setting, int kmax) {
    TpGeom t;
    const int64_t cl = chunk < n ? chunk : n;
    const int64_t nch = (n + cl - 1) / cl;
    const int64_t nsl = (cl + kSliceRows - 1) / kSliceRows;
    int cb = col_bits_setting;
    if (cb == 0) {
        const int want = kmax > 16 ? kDefaultColBits32 : kDefaultColBits;
        cb = 4;
        while (cb < want && (1ll << cb) < cl) ++cb;
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

bool args_ok(const void *rowptr, const int32_t *colidx, int64_t n, int32_t k, double slack,
             int64_t chunk, int32_t R) {
    if (!rowptr || !colidx) return false;
    if (n < 1 || n > (int64_t)INT32_MAX) return false;
    if (k < 1 || k > GREM_MAX_K) return false;
    if (chunk < 1 || R < 0) return false;
    if (!(slack >= 1.0) || std::isinf(slack)) return false;
    return true;
}

// ---- launch bracket: optional event pair per launch, error check after it --------------------------
struct Launcher {
    hipStream_t stream;
    int level = 0;                           // snapshot of the profiling level for this call
    int err = GREM_OK;
    hipEvent_t get_event() {
        {
            std::lock_guard<std::mutex> lock(g.mu);
            if (!g.pool.empty()) { hipEvent_t e = g.pool.back(); g.pool.pop_back(); return e; }
        }
        hipEvent_t e;
        // timing only: no system-scope fence (and the cache write-back it implies) when the event completes
        if (hipEventCreateWithFlags(&e, hipEventDisableSystemFence) != hipSuccess) { err = GREM_ERR_HIP; return nullptr; }
        return e;
    }
    template <typename F> void run(int cls, F &&f) {
        if (err) return;
        hipEvent_t a = nullptr, b = nullptr;
        if (level >= 2) {
            a = get_event(); b = get_event();
            if (err) return;
            if (hipEventRecord(a, stream) != hipSuccess) { err = GREM_ERR_HIP; return; }
        }
        f();
        if (hipGetLastError() != hipSuccess) { err = GREM_ERR_HIP; return; }
        if (level >= 2) {
            if (hipEventRecord(b, stream) != hipSuccess) { err = GREM_ERR_HIP; return; }
            std::lock_guard<std::mutex> lock(g.mu);
            g.events.push_back({cls, a, b});
        }
    }
    void mark() {
        if (err || level < 1) return;
        hipEvent_t e = get_event();
        if (err) return;
        if (hipEventRecord(e, stream) != hipSuccess) { err = GREM_ERR_HIP; return; }
        std::lock_guard<std::mutex> lock(g.mu);
        g.marks.push_back(e);
    }
    bool memset(void *p, int v, size_t bytes) {
        if (err) return false;
        if (bytes && hipMemsetAsync(p, v, bytes, stream) != hipSuccess) { err = GREM_ERR_HIP; return false; }
        return true;
    }
    bool read_back(void *host, const void *dev, size_t bytes) {
        if (err) return false;
        if (hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, stream) != hipSuccess ||
            hipStreamSynchronize(stream) != hipSuccess) { err = GREM_ERR_HIP; return false; }
        return true;
    }
};

bool set_lds(const void *f, size_t bytes) {
    return bytes <= 64 * 1024 ||
           hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) == hipSuccess;
}

// ======================================================================================================
// The re-laid-out copy of a graph's entries (two-phase route)
// ======================================================================================================
struct PlanData {
    const void *rowptr = nullptr;
    int rowptr_bits = 0;
    int64_t n = 0, nnz = 0;
    int hub_degree = 0;
    TpGeom geo;
    SweepPlan pl{};
    TpTables tb{};
    uint32_t *T = nullptr;
    uint16_t *R = nullptr;
    u64 *pmisc = nullptr;
    size_t slots = 0;
    unsigned long long maxdeg = 0, hub_entries = 0, total_hubs = 0, max_chunk_hubs = 0;
    bool have_degrees = false;              // maxdeg and nnz have been read back
    std::vector<uint32_t> nvs;              // hub shares per chunk (host copy of pl.ch_nvs)
    std::vector<uint32_t> chunk_hubs;       // hubs per chunk (host copy of pl.ch_nh)
    std::vector<u64> chunk_hub0;            // hubs of the chunks before it (host copy of pl.ch_hub0)
    int share_hubs = 0;
    int max_k = 0;                          // largest k whose score workgroups fit the LDS
    int lookup_target = 512;
};

// Sizes of the plan's pieces as functions of what is known at each stage; the same functions serve the
// real carve and the workspace bound.
struct PlanDims {
    int64_t n, nnz;
    TpGeom geo;
    size_t G;                       // slices of all chunks
    size_t hubs;                    // hubs of all chunks (or a bound)
    int npr, nps;
    int nr;                         // rows per chunk: slices, then the most hub shares any chunk has
    size_t slots;
};

size_t plan_slots(int64_t nnz, const TpGeom &geo, int nr) {
    // every sub-segment is padded to a multiple of kSubPad tuples
    const size_t subs = (size_t)geo.nch * (size_t)nr * (size_t)geo.nblk;
    return (size_t)(nnz > 0 ? nnz : 0) + (kSubPad - 1) * subs;
}

void plan_stage1(Carver &c, const PlanDims &d, SweepPlan &pl, u64 *&pmisc) {
    const size_t nch = (size_t)d.geo.nch;
    c.take(pl.sl_reg_cnt, d.G);
    c.take(pl.sl_reg_start, d.G);
    c.take(pl.sl_nh, d.G);
    c.take(pl.sl_hub_start, d.G);
    c.take(pl.sl_hent, d.G);
    c.take(pl.sl_hent_start, d.G);
    c.take(pl.sl_part_reg0, d.G * (size_t)kPlanParts);
    c.take(pl.share_h0, d.G);
    c.take(pl.share_nhs, d.G);
    c.take(pl.ch_regtot, nch);
    c.take(pl.ch_nh, nch);
    c.take(pl.ch_H, nch);
    c.take(pl.ch_nvs, nch);
    c.take(pl.ch_hbase, nch + 1);
    c.take(pl.ch_reg0, nch + 1);
    c.take(pl.ch_hub0, nch + 1);
    c.take(pmisc, 16);
}

void plan_stage2(Carver &c, const PlanDims &d, SweepPlan &pl) {
    c.take(pl.hub_row, d.hubs + 1);
    c.take(pl.hub_off, d.hubs + (size_t)d.geo.nch + 1);
}

void plan_stage3(Carver &c, const PlanDims &d, TpTables &tb, uint32_t *&T, uint16_t *&R) {
    const size_t segs = (size_t)d.geo.nch * (size_t)d.geo.nblk;
    const size_t rows = (size_t)d.geo.nch * (size_t)d.nr;
    c.take(tb.ta, segs * ((size_t)d.nr + 1));
    c.take(tb.dd, segs * (size_t)d.nr);
    c.take(tb.tstart, segs + 1);
    c.take(tb.sstart, rows + 1);
    c.take(tb.lo, d.G * (size_t)d.npr * ((size_t)d.geo.ngroups + 1));
    c.take(tb.loh, d.G * (size_t)d.nps * ((size_t)d.geo.ngroups + 1));
    c.take(tb.ustart, d.G * (size_t)d.npr);
    c.take(tb.ustart_h, d.G * (size_t)d.nps);
    uint8_t *t8 = nullptr;
    c.take(t8, d.slots * 3 + 16);            // 24 bytes per group of eight tuples: their place in Lx, their columns
    T = reinterpret_cast<uint32_t *>(t8);
    c.take(R, d.slots + 8);                  // row field, 2 bytes per tuple
}

// Builds the plan for (rowptr, colidx, n, chunk) under `o`.  `keep` receives what the plan consists
// of, `temp` the intermediate copy (given back before the function returns).  strict: a graph the
// route cannot take is GREM_ERR_ARG; otherwise the function returns GREM_OK with P.T == nullptr and the
// caller takes the plain route (P.maxdeg and P.nnz are valid once P.have_degrees is set).
// k: the number of partitions of the run the plan is built for, or 0 for any k up to 16 (then
// P.max_k says how far the plan reaches).
template <typename RowT>
int build_plan(PlanData &P, const RowT *rowptr, const int32_t *colidx, int64_t n, int64_t chunk, int32_t k,
               const Opts &o, Arena &keep, Arena &temp, Launcher &L, bool strict) {
    hipStream_t stream = L.stream;
    const int kmax = k ? k : o.plan_max_k;
    const TpGeom geo = tp_geometry(n, chunk, o.col_bits, kmax);
    if (!geo.ok) return GREM_ERR_ARG;            // (callers check the geometry first)
    const int hub_degree = o.hub_degree;
    P.rowptr = rowptr;
    P.rowptr_bits = (int)sizeof(RowT) * 8;
    P.n = n;
    P.hub_degree = hub_degree;
    P.geo = geo;
    PlanDims d{};
    d.n = n;
    d.geo = geo;
    d.G = (size_t)geo.nch * (size_t)geo.nsl;
    const int64_t cl = (int64_t)geo.chunk;
    const int nsl = geo.nsl;
    const unsigned G = (unsigned)d.G;
    SweepPlan &pl = P.pl;
    TpTables &tb = P.tb;

    // ---- stage 1: per slice and per chunk, regular entries, hubs, hub entries, shares
    if (!carve(keep, [&](Carver &c) { plan_stage1(c, d, pl, P.pmisc); })) return GREM_ERR_NOMEM;
    L.memset(P.pmisc, 0, 16 * 8);
    L.run(GREM_KERNEL_RELAYOUT, [&] {
        hipLaunchKernelGGL((k_plan_slices<RowT>), dim3(G), dim3(256), 0, stream, rowptr, n, cl, nsl,
                           (uint32_t)hub_degree, pl, P.pmisc);
    });
    L.run(GREM_KERNEL_RELAYOUT, [&] {
        hipLaunchKernelGGL(k_plan_chunks, dim3((unsigned)geo.nch), dim3(256), 0, stream, n, cl, nsl, geo.nblk,
                           (uint32_t)(kmax > 16 ? kHubsPerShare32 : kHubsPerShare16), pl, P.pmisc);
    });
    L.run(GREM_KERNEL_RELAYOUT, [&] {
        hipLaunchKernelGGL(k_tp_scan, dim3(3), dim3(1024), 0, stream, pl.ch_hbase, (int64_t)geo.nch, pl.ch_reg0,
                           (int64_t)geo.nch, pl.ch_hub0, (int64_t)geo.nch);
    });
    unsigned long long h[16] = {0};
    if (!L.read_back(h, P.pmisc, sizeof(h))) return L.err;
    P.maxdeg = h[0];
    P.nnz = (int64_t)h[3];
    P.have_degrees = true;
    P.max_chunk_hubs = h[6];
    P.hub_entries = h[8];
    P.total_hubs = h[12];
    d.nnz = P.nnz;
    d.hubs = (size_t)P.total_hubs;

    // ---- stage 2: the chunks' hub lists, the hubs every share touches
    if (!carve(keep, [&](Carver &c) { plan_stage2(c, d, pl); })) return GREM_ERR_NOMEM;
    L.run(GREM_KERNEL_RELAYOUT, [&] {
        hipLaunchKernelGGL((k_plan_hubs<RowT>), dim3(G), dim3(256), 0, stream, rowptr, n, cl, nsl,
                           (uint32_t)hub_degree, pl);
    });
    L.run(GREM_KERNEL_RELAYOUT, [&] {
        hipLaunchKernelGGL(k_plan_shares, dim3((G + 255) / 256), dim3(256), 0, stream, n, cl, nsl, (int)G, pl,
                           P.pmisc);
    });
    P.nvs.assign((size_t)geo.nch, 0u);
    P.chunk_hubs.assign((size_t)geo.nch, 0u);
    P.chunk_hub0.assign((size_t)geo.nch + 1, 0ull);
    if (P.total_hubs != 0) {
        if (hipMemcpyAsync(P.nvs.data(), pl.ch_nvs, (size_t)geo.nch * 4, hipMemcpyDeviceToHost, stream) != hipSuccess ||
            hipMemcpyAsync(P.chunk_hubs.data(), pl.ch_nh, (size_t)geo.nch * 4, hipMemcpyDeviceToHost, stream) != hipSuccess ||
            hipMemcpyAsync(P.chunk_hub0.data(), pl.ch_hub0, ((size_t)geo.nch + 1) * 8, hipMemcpyDeviceToHost, stream) !=
                hipSuccess)
            return GREM_ERR_HIP;
        if (!L.read_back(h, P.pmisc, sizeof(h))) return L.err;
    } else if (L.err) {
        return L.err;
    }
    const int share_hubs = (int)h[5];
    P.share_hubs = share_hubs;

    // ---- does the route fit?  A score workgroup's LDS (two per CU fit when a share touches few hubs);
    // a share may touch kMaxShareHubs hubs; sub-segment offsets are 32-bit
    {
        auto score_fits = [&](int kk) {
            const size_t dyn = ((size_t)kSliceRows / 2 + (size_t)share_hubs * kk + 3 * (size_t)kk) * 4;
            if (kk <= 16) return dyn + (size_t)kSliceRows * 32 <= 150 * 1024;
            return geo.cb <= 16 && dyn + (size_t)kSliceRows * 64 <= 158 * 1024;    // (a byte per label in the look-up's LDS)
        };
        int max_k = kmax;
        while (max_k > 1 && !score_fits(max_k) && k == 0) --max_k;
        P.max_k = max_k;
        // (the index of a word of Lx -- eight labels -- travels in 32 bits of T)
        const bool fits = score_fits(max_k) && share_hubs <= kMaxShareHubs &&
                          plan_slots(P.nnz, geo, 2 * geo.nsl) < (1ull << 35) &&
                          h[7] + 8ull * (2ull * (unsigned long long)geo.nsl + 2) * geo.nblk < (1ull << 32);
        if (!fits) return strict ? GREM_ERR_ARG : GREM_OK;
    }

    // ---- stage 3: shapes of the re-layout kernels, then the tables and streams
    // step 1 collects a unit's tuples in LDS: cut the slices (shares) in as many parts as it takes for
    // the largest to fit, two workgroups per CU
    constexpr size_t kGroupLds = 79 * 1024, kPlaceLds = 52 * 1024;
    auto group_fixed = [&](bool share, int np) {
        return (tp_source_words(share, np, share_hubs) + (size_t)geo.nblk + (size_t)geo.ngroups + 1 + kTpThreads / 64) * 4;
    };
    auto group_cap = [&](bool share, int np) {
        const size_t fixed = group_fixed(share, np);
        return (uint32_t)(kGroupLds > fixed ? (kGroupLds - fixed) / 4 : 0);
    };
    int npr = 1, nps = 1;
    // ... and, if that takes no more than kMaxParts, so small that a thread holds its share of the unit's
    // entries in registers (one round of kTpThreads * kTpBatch entries)
    const unsigned long long one_round = (unsigned long long)kTpThreads * kTpBatch;
    auto fits_unit = [&](bool share, int np, unsigned long long most, bool in_regs) {
        const unsigned long long unit = most / np + most / (8ull * np) + 64;
        return group_cap(share, np) >= unit && (!in_regs || unit <= one_round);
    };
    while (npr < kMaxParts && !fits_unit(false, npr, h[9], false)) npr *= 2;
    while (nps < kMaxParts && !fits_unit(true, nps, h[10], false)) nps += 1;
    {
        // slices differ in size: it is the average one whose parts should take one round (the larger ones
        // take two, and their tuples still fit LDS)
        const unsigned long long avg_slice =
            ((unsigned long long)P.nnz - P.hub_entries) / (unsigned long long)(d.G ? d.G : 1) + 1;
        int a = npr, b = nps;
        while (a < kMaxParts && !fits_unit(false, a, avg_slice, true)) a *= 2;
        while (b < kMaxParts && !fits_unit(true, b, h[10], true)) b += 1;
        if (fits_unit(false, a, avg_slice, true) && fits_unit(false, a, h[9], false)) npr = a;
        if (fits_unit(true, b, h[10], true)) nps = b;
    }
    d.npr = npr;
    d.nps = nps;
    const unsigned max_shares = (unsigned)h[11];            // no chunk has more hub shares than this
    d.nr = geo.nsl + (int)max_shares;
    d.slots = plan_slots(P.nnz, geo, d.nr);
    P.slots = d.slots;
    if (!carve(keep, [&](Carver &c) { plan_stage3(c, d, tb, P.T, P.R); })) { P.T = nullptr; return GREM_ERR_NOMEM; }
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
    tb.nr = d.nr;
    tb.nbc = geo.nbc;
    tb.nblk = geo.nblk;
    tb.cb = geo.cb;
    tb.flat = (tb.chunk_shift >= geo.cb && geo.chunk > 1) ? 1 : 0;
    tb.gb = geo.gb;
    tb.ngroups = geo.ngroups;
    tb.npr = npr;
    tb.nps = nps;
    P.lookup_target = geo.cb > 17 ? 256 : 512;

    const Arena::Mark tmark = temp.mark();
    const size_t subs = (size_t)geo.nch * (size_t)d.nr * (size_t)geo.nblk;
    uint32_t *U = (uint32_t *)temp.alloc((size_t)(P.nnz > 0 ? P.nnz : 0) * 4 + 16);
    tb.cnt = U ? (uint32_t *)temp.alloc(subs * 4) : nullptr;
    if (!U || !tb.cnt) { temp.release_to(tmark); P.T = nullptr; return GREM_ERR_NOMEM; }
    const u64 hub_base = (u64)P.nnz - P.hub_entries;        // U: the regular entries, then the hub streams

    const uint32_t capR = group_cap(false, npr), capS = group_cap(true, nps);
    const size_t groupR_lds = group_fixed(false, npr) + (size_t)capR * 4;
    const size_t groupS_lds = group_fixed(true, nps) + (size_t)capS * 4;
    // step 2: up to 8 slices at a time
    const int nbg = geo.nblk < (1 << geo.gb) ? geo.nblk : (1 << geo.gb);
    int batch = 8192 / nbg;
    if (batch > 8) batch = 8;
    if (batch < 1) batch = 1;
    {
        // ... and no more than fit the stage at the average row's size (a batch that does not fit is halved
        // by the kernel, at the price of setting its tables up again)
        const size_t fixed8 = tp_place_fixed_bytes(nbg, 8, 8 * (npr > nps ? npr : nps));
        const double cap8 = kPlaceLds > fixed8 ? (double)(kPlaceLds - fixed8) / 4.0 : 0.0;
        const double per_row = (double)d.slots / ((double)geo.nch * (double)d.nr) / (double)geo.ngroups;
        while (batch > 1 && per_row * 1.25 * batch > cap8) --batch;
    }
    const int maxruns = batch * (npr > nps ? npr : nps);
    const size_t place_fixed = tp_place_fixed_bytes(nbg, batch, maxruns);
    const uint32_t capP = (uint32_t)(kPlaceLds > place_fixed ? (kPlaceLds - place_fixed) / 4 : 0);
    const size_t place_lds = place_fixed + (size_t)capP * 4;
    L.memset(tb.cnt, 0, subs * 4);
    if (L.err || !set_lds((const void *)k_tp_group<RowT, false>, groupR_lds) ||
        !set_lds((const void *)k_tp_group<RowT, true>, groupS_lds) ||
        !set_lds((const void *)k_tp_place, place_lds)) {
        temp.release_to(tmark);
        P.T = nullptr;
        return GREM_ERR_HIP;
    }
    const unsigned segs = (unsigned)((int64_t)geo.nch * geo.nblk);
    L.run(GREM_KERNEL_RELAYOUT, [&] {
        hipLaunchKernelGGL((k_tp_group<RowT, false>), dim3(G * (unsigned)npr), dim3(kTpThreads), groupR_lds, stream,
                           rowptr, colidx, n, (uint32_t)hub_degree, pl, tb, share_hubs, capR, (int)nsl, U, hub_base);
    });
    // shares: no chunk has more than max_shares of them (none at all: nothing to launch)
    if (max_shares != 0)
        L.run(GREM_KERNEL_RELAYOUT, [&] {
            hipLaunchKernelGGL((k_tp_group<RowT, true>), dim3((unsigned)geo.nch * max_shares * (unsigned)nps),
                               dim3(kTpThreads), groupS_lds, stream, rowptr, colidx, n, (uint32_t)hub_degree, pl, tb,
                               share_hubs, capS, (int)max_shares, U, hub_base);
        });
    const unsigned rows_all = (unsigned)((int64_t)geo.nch * d.nr);
    L.run(GREM_KERNEL_RELAYOUT, [&] {
        hipLaunchKernelGGL(k_tp_scan_t, dim3((segs + 255) / 256), dim3(256), 0, stream, tb);
    });
    L.run(GREM_KERNEL_RELAYOUT, [&] {
        hipLaunchKernelGGL(k_tp_scan_d, dim3((rows_all + 255) / 256), dim3(256), 0, stream, tb);
    });
    L.run(GREM_KERNEL_RELAYOUT, [&] {
        hipLaunchKernelGGL(k_tp_scan, dim3(2), dim3(1024), 0, stream, tb.tstart, (int64_t)segs, tb.sstart,
                           (int64_t)rows_all, (u64 *)nullptr, (int64_t)0);
    });
    L.run(GREM_KERNEL_RELAYOUT, [&] {
        hipLaunchKernelGGL(k_tp_place, dim3((unsigned)((int64_t)geo.ngroups * geo.nch)), dim3(kPlaceThreads), place_lds,
                           stream, n, pl, tb, U, P.T, P.R, batch, capP);
    });
    temp.release_to(tmark);
    if (L.err) { P.T = nullptr; return L.err; }
    return GREM_OK;
}

// ======================================================================================================
// State of one run (Alg. 1's parts, sizes, nbr_counts and the admission tables)
// ======================================================================================================
template <typename LabelT> struct CallState {
    LabelT *Lc = nullptr, *prop = nullptr;
    long long *S = nullptr, *S2 = nullptr, *room = nullptr, *fillSorted = nullptr, *fillC = nullptr;
    uint32_t *cnt = nullptr, *tot = nullptr, *ocnt = nullptr;
    int32_t *fillRank = nullptr;
    unsigned long long *misc = nullptr;
    bool seed_complete = false;        // (host) the seed labels every vertex
};

template <typename LabelT>
void state_common(Carver &c, CallState<LabelT> &st, int64_t n, int64_t cl, int32_t k) {
    const size_t ntiles = (size_t)((cl + kAdmitTile - 1) / kAdmitTile);
    c.take(st.Lc, (size_t)n);
    c.take(st.prop, (size_t)cl);
    c.take(st.S, (size_t)k);
    c.take(st.S2, (size_t)k);                // the sizes' other copy (the one-launch spill reads one, writes the other)
    c.take(st.cnt, ntiles * (size_t)k);
    c.take(st.tot, 2 * (size_t)k);
    c.take(st.room, (size_t)k);
    c.take(st.ocnt, ntiles);
    c.take(st.fillRank, (size_t)k);
    c.take(st.fillSorted, (size_t)k);
    c.take(st.fillC, (size_t)k + 1);
    c.take(st.misc, 16);
}

// prepass: compact labels and sizes from the seed, its validity; with rowptr also the largest degree
template <typename RowT, typename LabelT>
void launch_prepass(Launcher &L, const RowT *rowptr_or_null, const int32_t *seed, int64_t n, int32_t k, long long P,
                    CallState<LabelT> &st) {
    hipStream_t stream = L.stream;
    L.memset(st.S, 0, (size_t)k * 8);
    L.memset(st.misc, 0, 16 * 8);
    int64_t blocks = (n + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    L.run(GREM_KERNEL_PREPASS, [&] {
        hipLaunchKernelGGL((k_prepass<RowT, LabelT>), dim3((unsigned)blocks), dim3(256), 0, stream, rowptr_or_null, seed,
                           n, (int)k, st.Lc, (unsigned long long *)st.S, st.misc);
    });
    if (seed)
        L.run(GREM_KERNEL_PREPASS, [&] {
            hipLaunchKernelGGL(k_check_seed_sizes, dim3((k + 255) / 256), dim3(256), 0, stream, st.S, (int)k, P, st.misc);
        });
}

template <typename LabelT>
void launch_spill(Launcher &L, CallState<LabelT> &st, int64_t lo, int64_t hi, int32_t k, unsigned admit_blocks) {
    hipStream_t stream = L.stream;
    L.run(GREM_KERNEL_SPILL_SCAN, [&] {
        hipLaunchKernelGGL(k_spill_scan, dim3(1), dim3(kScanThreads), 0, stream, st.ocnt, (int)admit_blocks, (int)k, st.S,
                           st.fillRank, st.fillSorted, st.fillC, st.misc);
    });
    L.run(GREM_KERNEL_SPILL_FILL, [&] {
        hipLaunchKernelGGL((k_spill_fill<LabelT>), dim3(admit_blocks), dim3(kAdmitThreads), (size_t)k * 4, stream, st.Lc, lo,
                           hi, (int)k, st.ocnt, st.fillRank, st.fillC, (unsigned long long *)st.S, st.misc);
    });
}

template <typename LabelT>
void launch_outputs(Launcher &L, CallState<LabelT> &st, int64_t n, int32_t k, int32_t *labels_out, int64_t *sizes_out) {
    hipStream_t stream = L.stream;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (labels_out)
        L.run(GREM_KERNEL_EXPAND, [&] {
            hipLaunchKernelGGL((k_expand<LabelT>), dim3((unsigned)blocks), dim3(256), 0, stream, st.Lc, n, labels_out);
        });
    if (sizes_out)
        L.run(GREM_KERNEL_EXPAND, [&] {
            hipLaunchKernelGGL(k_copy_sizes, dim3((k + 255) / 256), dim3(256), 0, stream, st.S, (int)k, sizes_out);
        });
}

// ---- two-phase route: per-call arrays beside the common state ---------------------------------------
struct TpState {
    uint32_t *Lx = nullptr, *Hhub = nullptr, *E32 = nullptr, *Ehub = nullptr;
    uint16_t *Rdyn = nullptr, *E16 = nullptr;
    uint8_t *Lc4 = nullptr;            // k <= 16: the labels two per byte, kept by the admission from the second pass on
    uint8_t *hub_old = nullptr;        // the labels of the chunk's hubs, by their place in its list (see k_admit_hubs)
    uint32_t *coarse = nullptr;        // two tables of the tiles' mover counts added up 32 tiles at a time (k_admit_hubs)
};

// twice: two tables of the chunk's hub counts and of the hubs' estimates (the admission that also does the
// hubs' part reads one and writes the other)
void state_two_phase(Carver &c, TpState &t, int64_t n, int32_t k, size_t slots, size_t max_chunk_hubs, size_t total_hubs,
                     bool seeded, bool use16, bool external_E, bool twice) {
    uint8_t *lx = nullptr;
    c.take(lx, (k <= 16 ? slots / 2 : slots) + 16);               // label, 4 bits per tuple (8 when k > 16)
    t.Lx = reinterpret_cast<uint32_t *>(lx);
    c.take(t.Hhub, (twice ? 2 : 1) * (max_chunk_hubs + 1) * (size_t)k);
    c.take(t.Rdyn, seeded ? slots + 8 : 0);                       // seeded runs: R with the unassigned neighbours marked
    c.take(t.E16, use16 ? (size_t)n * (size_t)k : 0);
    c.take(t.E32, (!use16 && !external_E) ? (size_t)n * (size_t)k : 0);
    c.take(t.Ehub, (use16 && !external_E) ? (twice ? 2 : 1) * (total_hubs + 1) * (size_t)k : 0);
    c.take(t.Lc4, k <= 16 ? (size_t)n / 2 + 16 : 0);
    c.take(t.hub_old, twice ? max_chunk_hubs + 16 : 0);
    c.take(t.coarse, twice ? 2 * (size_t)(kAdmitTilesMax / kCoarseTiles) * (size_t)k : 0);
}

// The admission kernel does the hubs' blend and proposal itself when every chunk has few hubs and few
// tiles and the hubs' estimates live in a table of their own (16-bit estimates, no caller's array).
bool admission_takes_hubs(const PlanData &P, bool use16, bool external_E) {
    const int64_t tiles = ((int64_t)P.geo.chunk + kAdmitTile - 1) / kAdmitTile;
    return use16 && !external_E && P.max_chunk_hubs <= (unsigned long long)kAdmitHubsMax && tiles <= kAdmitTilesMax;
}

// Alg. 1's loop on a plan.  `prepared`: the common state with the prepass run and the seed validated by
// the caller; otherwise this function does both (one read-back when there is a seed).
// fixed_labels: nothing is decided.  The seed is a labelling that stays as it is (R = 0, estimates_out
// given): after the initial look-up of every label, each chunk runs its counting launches only, and
// estimates_out receives cnt_nbrs (Alg. 2) of every vertex under that labelling.
template <typename RowT>
int run_two_phase(const PlanData &P, int32_t k, double slack, int32_t R, const int32_t *seed, int32_t *labels_out,
                  int64_t *sizes_out, uint32_t *estimates_out, Arena &mem, Launcher &L, CallState<uint8_t> *prepared,
                  bool fixed_labels = false) {
    hipStream_t stream = L.stream;
    const RowT *rowptr = (const RowT *)P.rowptr;
    const int64_t n = P.n;
    const TpGeom &geo = P.geo;
    const TpTables &tb = P.tb;
    const SweepPlan &pl = P.pl;
    const int64_t cl = (int64_t)geo.chunk;
    const long long cap = grem_capacity(n, k, slack);
    const bool external_E = estimates_out != nullptr;
    const int hub_degree = P.hub_degree;
    if (R >= 32 || (P.maxdeg << R) >= (1ull << 32)) return GREM_ERR_RANGE;
    if (external_E && (((uintptr_t)estimates_out) & 15u) != 0) return GREM_ERR_ARG;
    if (fixed_labels && (!seed || !external_E || R != 0)) return GREM_ERR_ARG;
    // estimates of the regular rows stay below hub_degree * 2^R: 16 bits when that fits
    // (the counts of a fixed labelling go straight to the caller's 32-bit array: no 16-bit copy to expand)
    const bool use16 = !fixed_labels && (((unsigned long long)(hub_degree - 1)) << R) <= 65535ull;

    const bool hubs_in_admission = admission_takes_hubs(P, use16, external_E);

    CallState<uint8_t> st;
    if (prepared) {
        st = *prepared;
    } else {
        if (!carve(mem, [&](Carver &c) { state_common(c, st, n, cl, k); })) return GREM_ERR_NOMEM;
    }
    TpState t;
    if (!carve(mem, [&](Carver &c) {
            state_two_phase(c, t, n, k, P.slots, (size_t)P.max_chunk_hubs, (size_t)P.total_hubs, seed != nullptr, use16,
                            external_E, hubs_in_admission);
        }))
        return GREM_ERR_NOMEM;
    if (!prepared) {
        launch_prepass<RowT, uint8_t>(L, (const RowT *)nullptr, seed, n, k, cap, st);
        if (seed) {
            unsigned long long h[16] = {0};
            if (!L.read_back(h, st.misc, sizeof(h))) return L.err;
            if (h[1] != 0 || h[2] != 0) return GREM_ERR_SEED;
            st.seed_complete = h[5] == 0;
        }
    }
    uint32_t *E32 = external_E ? estimates_out : t.E32;
    uint32_t *Ehub_rows = (use16 && !external_E) ? nullptr : E32;    // hubs: rows of E32 when there is one, else Ehub
    if (k > P.max_k) return GREM_ERR_ARG;
    const bool wide = k > 16;                     // 8-bit labels in Lx, 128 KB of counters per slice
    const size_t score_lds = ((size_t)kSliceRows / 2 + (size_t)P.share_hubs * k + 3 * (size_t)k) * 4 +
                             (wide ? (size_t)kSliceRows * 64 : 0);
    const size_t lookup_lds = wide ? ((size_t)1 << (geo.cb > 4 ? geo.cb : 4)) : ((size_t)1 << (geo.cb > 5 ? geo.cb - 1 : 4));
    if (wide) {
        if (!set_lds((const void *)k_tp_lookup<true, false, 8>, lookup_lds) ||
            !set_lds((const void *)k_tp_lookup<true, true, 8>, lookup_lds) ||
            !set_lds((const void *)k_tp_score<uint32_t, 32>, score_lds) ||
            !set_lds((const void *)k_tp_score<uint16_t, 32>, score_lds))
            return GREM_ERR_HIP;
    } else {
        if (!set_lds((const void *)k_tp_lookup<true, false, 4>, lookup_lds) ||
            !set_lds((const void *)k_tp_lookup<true, true, 4>, lookup_lds) ||
            !set_lds((const void *)k_tp_score<uint32_t, 16>, score_lds) ||
            !set_lds((const void *)k_tp_score<uint16_t, 16>, score_lds) ||
            !set_lds((const void *)k_tp_score<uint32_t, 16, true>, score_lds) ||
            !set_lds((const void *)k_tp_score<uint16_t, 16, true>, score_lds))
            return GREM_ERR_HIP;
    }
    L.memset(t.Hhub, 0, (hubs_in_admission ? 2 : 1) * ((size_t)P.max_chunk_hubs + 1) * (size_t)k * 4);
    const size_t coarse_row = (size_t)(kAdmitTilesMax / kCoarseTiles) * (size_t)k;
    if (hubs_in_admission) L.memset(t.coarse, 0, 2 * coarse_row * 4);

    // look-ups of the labels of chunks [c0, c0 + count): shares per column block sized so that one
    // launch fills the chip without cutting the blocks' streams into crumbs
    // `mark`: seeded runs, first pass: the row fields the score kernels read are those of Rdyn, where
    // bit 0 also marks the tuples whose neighbour is unassigned (set by the initial look-up from global
    // memory, cleared by the look-up of the neighbour's chunk)
    auto lookup = [&](int c0, int count, int cmin, bool from_lds, bool mark, const uint8_t *labels4 = nullptr) {
        if (cmin >= geo.nch) return;
        const int64_t per_block = P.nnz / geo.nblk + 1;
        int spb = P.lookup_target / geo.nbc;
        const int64_t by_work = per_block / 8192 + 1;
        if (spb > by_work) spb = (int)by_work;
        if (spb < 1) spb = 1;
        const dim3 grid((unsigned)(geo.nbc * spb), (unsigned)count);
        auto go = [&](auto kernel, size_t lds) {
            hipLaunchKernelGGL(kernel, grid, dim3(kTpThreads), lds, stream, P.T, t.Lx, P.R, t.Rdyn, tb,
                               (const uint8_t *)st.Lc, labels4, n, c0, cmin, spb);
        };
        L.run(GREM_KERNEL_LOOKUP, [&] {
            if (wide) {
                if (!from_lds) go(k_tp_lookup<false, true, 8>, 0);
                else if (mark) go(k_tp_lookup<true, true, 8>, lookup_lds);
                else go(k_tp_lookup<true, false, 8>, lookup_lds);
            } else {
                if (!from_lds) go(k_tp_lookup<false, true, 4>, 0);
                else if (mark) go(k_tp_lookup<true, true, 4>, lookup_lds);
                else go(k_tp_lookup<true, false, 4>, lookup_lds);
            }
        });
    };
    // A seed that leaves vertices without a label: the first pass reads its row fields from Rdyn, where the
    // initial look-up marks the tuples whose neighbour has none.  A seed that labels every vertex marks
    // nothing: R serves as it is, and the initial look-up is the one that copies the labels to LDS.
    const bool marks = seed != nullptr && !st.seed_complete;
    if (seed) {        // the seeds are the labels every first-pass look-up starts from
        for (int c0 = 0; c0 < geo.nch; c0 += 32768) {
            const int count = geo.nch - c0 < 32768 ? geo.nch - c0 : 32768;
            lookup(c0, count, 0, !marks, marks);
        }
    }
    L.mark();
    const size_t max_chunk_hubs = (size_t)P.max_chunk_hubs;
    uint32_t prev_hubs = 0;                 // hubs of the chunk before (whose counts the admission clears)
    // first pass, chunks of at most kSpillSmallTiles tiles: the spill is one launch that reads the sizes from one
    // array and writes them to the other; the two take turns from chunk to chunk
    const bool spill_small = (cl + kAdmitTile - 1) / kAdmitTile <= kSpillSmallTiles;
    long long *Snow = st.S;
    for (int pass = 0; pass <= R && !L.err; ++pass) {
        for (int64_t c = 0; c < geo.nch && !L.err; ++c) {
            const int64_t lo = c * cl;
            const int64_t hi = (lo + cl < n) ? lo + cl : n;
            const int64_t len = hi - lo;
            const unsigned admit_blocks = (unsigned)((len + kAdmitTile - 1) / kAdmitTile);
            const unsigned blocks = (unsigned)((len + kSliceRows - 1) / kSliceRows);
            const int jlim = (pass == 0 && !seed) ? (int)c * geo.nbc : geo.nblk;
            // the estimates are state between passes and, if the caller asked for them, output: the last
            // pass does not store them otherwise
            const int store_e = (pass < R || external_E) ? 1 : 0;
            const uint16_t *rows_now = (marks && pass == 0) ? t.Rdyn : P.R;
            // from the second pass on every vertex has a label before its chunk's admission, which then
            // also leaves the chunk's labels two per byte for the look-ups (chunk starts must be even)
            uint8_t *packed_now = (pass >= 1 && t.Lc4 && (cl & 1) == 0) ? t.Lc4 : nullptr;
            const int64_t step = (int64_t)pass * geo.nch + c;
            uint32_t *Hnow = t.Hhub + (hubs_in_admission ? (size_t)(step & 1) * ((size_t)max_chunk_hubs + 1) * (size_t)k : 0);
            auto score = [&](auto kernel, auto *Eptr) {
                hipLaunchKernelGGL(kernel, dim3(blocks), dim3(kTpThreads), score_lds, stream, rows_now, t.Lx, tb, pl,
                                   (const uint8_t *)st.Lc, Snow, Eptr, Hnow, (uint8_t *)st.prop, st.cnt, st.room, (int)c,
                                   lo, hi, (int)k, jlim, P.share_hubs, P.nvs[(size_t)c], pass, cap, store_e,
                                   hubs_in_admission ? t.hub_old : (uint8_t *)nullptr,
                                   hubs_in_admission ? t.coarse + (size_t)(step & 1) * coarse_row : (uint32_t *)nullptr);
            };
            L.run(GREM_KERNEL_SCORE, [&] {
                if (wide) {
                    if (use16) score(k_tp_score<uint16_t, 32>, t.E16);
                    else score(k_tp_score<uint32_t, 32>, E32);
                } else {
                    // (k <= 8: a row's few counters spread over the LDS banks)
                    if (k <= 8) {
                        if (use16) score(k_tp_score<uint16_t, 16, true>, t.E16);
                        else score(k_tp_score<uint32_t, 16, true>, E32);
                    } else {
                        if (use16) score(k_tp_score<uint16_t, 16>, t.E16);
                        else score(k_tp_score<uint32_t, 16>, E32);
                    }
                }
            });
            if (hubs_in_admission) {
                // one launch: every workgroup works out the chunk's hubs for itself; two tables of hub counts
                // take turns from chunk to chunk, two tables of hub estimates from pass to pass
                const size_t hrow = (size_t)max_chunk_hubs + 1, erow = (size_t)P.total_hubs + 1;
                const uint32_t nh = P.chunk_hubs[(size_t)c];
                const size_t hub0 = (size_t)P.chunk_hub0[(size_t)c];
                uint32_t *Hother = t.Hhub + (size_t)((step + 1) & 1) * hrow * (size_t)k;
                const uint32_t *Eold = t.Ehub + ((size_t)((pass + 1) & 1) * erow + hub0) * (size_t)k;
                uint32_t *Enew = t.Ehub + ((size_t)(pass & 1) * erow + hub0) * (size_t)k;
                L.run(GREM_KERNEL_APPLY, [&] {
                    const dim3 grid((admit_blocks + kSmallApplyTiles - 1) / kSmallApplyTiles);
                    auto go = [&](auto kernel) {
                        hipLaunchKernelGGL(kernel, grid, dim3(kAdmitTile), 0, stream, (uint8_t *)st.Lc, (const uint8_t *)st.prop,
                                           lo, hi, (int)k, (const uint32_t *)st.cnt, (int)admit_blocks,
                                           (const long long *)st.room, (unsigned long long *)Snow, st.ocnt, pass, packed_now,
                                           (const int32_t *)(pl.hub_row + hub0), (const uint8_t *)t.hub_old, nh,
                                           (const uint32_t *)Hnow, Hother,
                                           prev_hubs, Eold, Enew, store_e,
                                           (const uint32_t *)(t.coarse + (size_t)(step & 1) * coarse_row),
                                           t.coarse + (size_t)((step + 1) & 1) * coarse_row);
                    };
                    if (wide) go(k_admit_hubs<32>);
                    else go(k_admit_hubs<16>);
                });
                prev_hubs = nh;
            } else {
            // (one workgroup more than the hubs need: it adds up the chunk's mover counts)
            L.run(GREM_KERNEL_HUBS, [&] {
                if (wide)
                    hipLaunchKernelGGL(k_hub_finalize<32>, dim3((unsigned)((max_chunk_hubs + 7) / 8) + 1), dim3(256), 0,
                                       stream, pl, (const uint8_t *)st.Lc, st.room, Ehub_rows, t.Ehub, t.Hhub,
                                       (uint8_t *)st.prop, st.cnt, (int)c, lo, (int)k, pass, store_e, (int)admit_blocks,
                                       st.tot);
                else
                    hipLaunchKernelGGL(k_hub_finalize<16>, dim3((unsigned)((max_chunk_hubs + 15) / 16) + 1), dim3(256), 0,
                                       stream, pl, (const uint8_t *)st.Lc, st.room, Ehub_rows, t.Ehub, t.Hhub,
                                       (uint8_t *)st.prop, st.cnt, (int)c, lo, (int)k, pass, store_e, (int)admit_blocks,
                                       st.tot);
            });
            if (fixed_labels) continue;          // counts only: nothing to admit, no new labels to look up
            // admission: the score kernel has counted the movers per tile and taken the sizes' snapshot, and
            // the tiles are few enough that every workgroup adds up the earlier tiles' counts itself
            L.run(GREM_KERNEL_APPLY, [&] {
                const dim3 grid((admit_blocks + kSmallApplyTiles - 1) / kSmallApplyTiles);
                if (wide)
                    hipLaunchKernelGGL(k_apply_small<32>, grid, dim3(kAdmitTile), 0, stream, (uint8_t *)st.Lc,
                                       (const uint8_t *)st.prop, lo, hi, (int)k, st.cnt, st.room, st.tot,
                                       (unsigned long long *)Snow, st.ocnt, pass, (uint8_t *)nullptr);
                else
                    hipLaunchKernelGGL(k_apply_small<16>, grid, dim3(kAdmitTile), 0, stream, (uint8_t *)st.Lc,
                                       (const uint8_t *)st.prop, lo, hi, (int)k, st.cnt, st.room, st.tot,
                                       (unsigned long long *)Snow, st.ocnt, pass, packed_now);
            });
            }
            if (pass == 0) {
                if (spill_small) {
                    long long *Snext = Snow == st.S ? st.S2 : st.S;
                    L.run(GREM_KERNEL_SPILL_FILL, [&] {
                        const dim3 grid((admit_blocks + kSmallApplyTiles - 1) / kSmallApplyTiles);
                        if (wide)
                            hipLaunchKernelGGL(k_spill_small<32>, grid, dim3(kAdmitTile), 0, stream, (uint8_t *)st.Lc, lo, hi,
                                               (int)k, (const uint32_t *)st.ocnt, (int)admit_blocks, (const long long *)Snow,
                                               Snext);
                        else
                            hipLaunchKernelGGL(k_spill_small<16>, grid, dim3(kAdmitTile), 0, stream, (uint8_t *)st.Lc, lo, hi,
                                               (int)k, (const uint32_t *)st.ocnt, (int)admit_blocks, (const long long *)Snow,
                                               Snext);
                    });
                    Snow = Snext;
                } else {
                    launch_spill<uint8_t>(L, st, lo, hi, k, admit_blocks);
                }
            }
            // the chunk's new labels, looked up for every row that will read them: rows of later chunks in
            // this pass, rows of this and earlier chunks in the next pass (if there is one)
            lookup((int)c, 1, pass == R ? (int)c + 1 : 0, true, marks && pass == 0, packed_now);
        }
        L.mark();
    }
    st.S = Snow;
    launch_outputs<uint8_t>(L, st, n, k, labels_out, sizes_out);
    if (use16 && external_E) {
        int64_t blocks = (n + 255) / 256;
        if (blocks > 256 * 32) blocks = 256 * 32;
        L.run(GREM_KERNEL_EXPAND, [&] {
            hipLaunchKernelGGL((k_expand_estimates<RowT>), dim3((unsigned)blocks), dim3(256), 0, stream, rowptr, n, (int)k,
                               (uint32_t)hub_degree, t.E16, estimates_out);
        });
    }
    L.mark();
    return L.err;
}

// ---- plain route ------------------------------------------------------------------------------------
struct PlainExtra {
    uint32_t *E = nullptr, *long_cnt = nullptr, *long_list = nullptr;
};

void state_plain(Carver &c, PlainExtra &x, int64_t n, int64_t cl, int32_t k, int64_t nchunks, bool external_E) {
    c.take(x.E, external_E ? 0 : (size_t)n * (size_t)k);
    c.take(x.long_cnt, (size_t)nchunks);
    c.take(x.long_list, (size_t)cl);
}

// Alg. 1's loop straight on the CSR.  `st` is prepared (prepass run, seed and degrees validated).
template <typename RowT, typename LabelT>
int run_plain(const RowT *rowptr, const int32_t *colidx, int64_t n, int32_t k, double slack, int64_t cl, int32_t R,
              const int32_t *seed, int32_t *labels_out, int64_t *sizes_out, uint32_t *estimates_out, const Opts &o,
              unsigned long long maxdeg, Arena &mem, Launcher &L, CallState<LabelT> &st) {
    hipStream_t stream = L.stream;
    const long long P = grem_capacity(n, k, slack);
    const bool external_E = estimates_out != nullptr;
    const int64_t nchunks = (n + cl - 1) / cl;
    const bool use_lds = o.hist_mode != GREM_HIST_GLOBAL && k <= kLdsMaxK;
    PlainExtra x;
    if (!carve(mem, [&](Carver &c) { state_plain(c, x, n, cl, k, nchunks, external_E); })) return GREM_ERR_NOMEM;
    uint32_t *E = external_E ? estimates_out : x.E;

    // tile shape of the score kernels
    int tv = kGlobalTile;
    if (use_lds) {
        tv = 256;
        while (tv > 1 && (size_t)tv * k * 4 > (size_t)kLdsHistBytes) tv >>= 1;
    }
    if (maxdeg * (unsigned long long)tv >= (1ull << 31)) return GREM_ERR_RANGE;
    const size_t score_lds = use_lds ? ((size_t)tv * k + tv + 1 + k) * 4 : ((size_t)tv + 1 + k) * 4;
    const size_t count_lds = (size_t)k * 4;
    const size_t apply_lds = ((size_t)k + (size_t)(kAdmitThreads / 64) * k + 2 * (size_t)k) * 4;
    if (!set_lds((const void *)k_apply<LabelT, false>, apply_lds)) return GREM_ERR_HIP;

    // rows this long are taken out of their tile and spread over a grid of their own
    const bool split_long = maxdeg >= (unsigned long long)o.long_row_degree;
    const size_t long_lds = (size_t)k * 4;
    if (split_long && !set_lds((const void *)k_long_rows<RowT, LabelT>, long_lds)) return GREM_ERR_HIP;

    L.mark();
    for (int pass = 0; pass <= R && !L.err; ++pass) {
        if (split_long) L.memset(x.long_cnt, 0, (size_t)nchunks * 4);
        for (int64_t c = 0; c < nchunks && !L.err; ++c) {
            const int64_t lo = c * cl;
            const int64_t hi = (lo + cl < n) ? lo + cl : n;
            const int64_t len = hi - lo;
            const int64_t gather_limit = (pass == 0 && !seed) ? lo : n;
            const unsigned admit_blocks = (unsigned)((len + kAdmitTile - 1) / kAdmitTile);
            const LongRows lr{split_long ? (uint32_t)o.long_row_degree : 0xFFFFFFFFu, kLongRowPart, x.long_cnt + c,
                              x.long_list};
            const unsigned score_blocks = (unsigned)((len + tv - 1) / tv);
            L.run(GREM_KERNEL_SCORE, [&] {
                if (use_lds)
                    hipLaunchKernelGGL((k_score_lds<RowT, LabelT>), dim3(score_blocks), dim3(kScoreThreads), score_lds,
                                       stream, rowptr, colidx, st.Lc, st.S, E, st.prop, lo, hi, (int)k, tv, pass, P,
                                       gather_limit, lr);
                else
                    hipLaunchKernelGGL((k_score_global<RowT, LabelT>), dim3(score_blocks), dim3(kScoreThreads), score_lds,
                                       stream, rowptr, colidx, st.Lc, st.S, E, st.prop, lo, hi, (int)k, pass, P,
                                       gather_limit, lr);
            });
            if (split_long) {
                L.run(GREM_KERNEL_HUBS, [&] {
                    hipLaunchKernelGGL((k_long_rows<RowT, LabelT>), dim3(kLongRowGrid), dim3(kScoreThreads), long_lds, stream,
                                       rowptr, colidx, st.Lc, E, (int)k, pass, gather_limit, lr);
                });
                L.run(GREM_KERNEL_HUBS, [&] {
                    hipLaunchKernelGGL((k_long_propose<LabelT>), dim3(64), dim3(64), 0, stream, st.Lc, st.S, E, st.prop, lo,
                                       (int)k, pass, P, lr);
                });
            }
            // admission: per-tile mover counts, their prefix over the tiles, ranks
            L.run(GREM_KERNEL_COUNT, [&] {
                hipLaunchKernelGGL((k_count<LabelT>), dim3(admit_blocks), dim3(kAdmitThreads), count_lds, stream, st.Lc,
                                   st.prop, lo, hi, (int)k, st.cnt);
            });
            L.run(GREM_KERNEL_SCAN, [&] {
                hipLaunchKernelGGL(k_scan, dim3(1), dim3(kScanThreads), 0, stream, st.cnt, (int)admit_blocks, (int)k, st.S,
                                   P, st.room);
            });
            L.run(GREM_KERNEL_APPLY, [&] {
                hipLaunchKernelGGL((k_apply<LabelT, false>), dim3(admit_blocks), dim3(kAdmitThreads), apply_lds, stream,
                                   st.Lc, st.prop, lo, hi, (int)k, st.cnt, st.room, (unsigned long long *)st.S, st.ocnt,
                                   pass);
            });
            if (pass == 0) launch_spill<LabelT>(L, st, lo, hi, k, admit_blocks);
        }
        L.mark();
    }
    launch_outputs<LabelT>(L, st, n, k, labels_out, sizes_out);
    L.mark();
    return L.err;
}

size_t plain_bytes(int64_t n, int32_t k, int64_t cl, bool external_E) {
    const int64_t nchunks = (n + cl - 1) / cl;
    PlainExtra x;
    size_t a;
    if (k <= 255) {
        CallState<uint8_t> st;
        a = carve_size([&](Carver &c) { state_common(c, st, n, cl, k); });
    } else {
        CallState<uint16_t> st;
        a = carve_size([&](Carver &c) { state_common(c, st, n, cl, k); });
    }
    return a + carve_size([&](Carver &c) { state_plain(c, x, n, cl, k, nchunks, external_E); });
}

// One partition call: route choice, memory, validation, then one of the two loops.
template <typename RowT, typename LabelT>
int run_partition(const RowT *rowptr, const int32_t *colidx, int64_t n, int32_t k, double slack, int64_t chunk,
                  int32_t R, const int32_t *seed, int32_t *labels_out, int64_t *sizes_out, uint32_t *estimates_out,
                  const Opts &o, hipStream_t stream) {
    const int64_t cl = chunk < n ? chunk : n;             // a chunk longer than the graph is the whole graph
    const long long P = grem_capacity(n, k, slack);
    const bool external_E = estimates_out != nullptr;
    if (o.hist_mode == GREM_HIST_LDS && k > kLdsMaxK) return GREM_ERR_ARG;
    const bool forced = o.hist_mode == GREM_HIST_SWEEP;
    bool try_sweep = false;
    if constexpr (sizeof(LabelT) == 1) {
        const TpGeom geo = tp_geometry(n, cl, o.col_bits, k);
        const bool can = k <= kSweepMaxK && geo.ok && (((uintptr_t)estimates_out) & 15u) == 0;
        if (forced && !can) return GREM_ERR_ARG;
        try_sweep = can && (forced || (o.hist_mode == GREM_HIST_AUTO && n >= kSweepMinN && cl >= kSweepMinChunk));
    } else {
        if (forced) return GREM_ERR_ARG;
    }

    Arena mem;
    mem.stream = stream;
    Launcher L{stream};
    {
        std::lock_guard<std::mutex> lock(g.mu);
        mem.base = (char *)g.ws;
        mem.cap = g.ws_bytes;
        L.level = g.prof_level;
    }
    if (mem.base && mem.cap < plain_bytes(n, k, cl, external_E)) return GREM_ERR_NOMEM;
    L.mark();

    CallState<LabelT> st;
    if (!carve(mem, [&](Carver &c) { state_common(c, st, n, cl, k); })) { mem.release_all(); return GREM_ERR_NOMEM; }
    unsigned long long maxdeg = 0;
    int rc = GREM_OK;
    bool done = false;
    if constexpr (sizeof(LabelT) == 1) {
        if (try_sweep) {
            // the plan's first kernels also find the largest degree, so the prepass leaves the rows alone
            launch_prepass<RowT, LabelT>(L, (const RowT *)nullptr, seed, n, k, P, st);
            const Arena::Mark before_plan = mem.mark();
            PlanData plan;
            rc = build_plan<RowT>(plan, rowptr, colidx, n, cl, k, o, mem, mem, L, forced);
            if (rc == GREM_ERR_NOMEM && !forced) {       // (a workspace that holds the plain route's state only)
                rc = GREM_OK;
                plan.T = nullptr;
            }
            if (rc != GREM_OK) { mem.release_all(); return rc; }
            if (plan.have_degrees) {
                maxdeg = plan.maxdeg;
                if (seed) {
                    unsigned long long h[16] = {0};
                    if (!L.read_back(h, st.misc, sizeof(h))) { mem.release_all(); return L.err; }
                    if (h[1] != 0 || h[2] != 0) { mem.release_all(); return GREM_ERR_SEED; }
                    st.seed_complete = h[5] == 0;
                }
                if (R >= 32 || (maxdeg << R) >= (1ull << 32)) { mem.release_all(); return GREM_ERR_RANGE; }
            } else {
                try_sweep = false;                       // the plain route's own prepass finds the degrees
            }
            if (plan.T) {
                rc = run_two_phase<RowT>(plan, k, slack, R, seed, labels_out, sizes_out, estimates_out, mem, L, &st);
                if (rc == GREM_ERR_NOMEM && !forced) rc = GREM_OK;      // nothing of the loop is enqueued yet
                else done = true;
            }
            if (!done) mem.release_to(before_plan);
        }
    }
    if (!done) {
        if (!try_sweep) {
            launch_prepass<RowT, LabelT>(L, rowptr, seed, n, k, P, st);
            unsigned long long h[16] = {0};
            if (!L.read_back(h, st.misc, sizeof(h))) { mem.release_all(); return L.err; }
            if (h[1] != 0 || h[2] != 0) { mem.release_all(); return GREM_ERR_SEED; }
            maxdeg = h[0];
            if (R >= 32 || (maxdeg << R) >= (1ull << 32)) { mem.release_all(); return GREM_ERR_RANGE; }
        }
        rc = run_plain<RowT, LabelT>(rowptr, colidx, n, k, slack, cl, R, seed, labels_out, sizes_out, estimates_out, o,
                                     maxdeg, mem, L, st);
    }
    mem.release_all();
    return rc;
}

template <typename RowT>
int dispatch_labels(const RowT *rowptr, const int32_t *colidx, int64_t n, int32_t k, double slack,
                    int64_t chunk, int32_t R, const int32_t *seed, int32_t *labels_out,
                    int64_t *sizes_out, uint32_t *estimates_out, const grem_options *options, void *stream) {
    if (!args_ok(rowptr, colidx, n, k, slack, chunk, R) || !labels_out) return GREM_ERR_ARG;
    Opts o;
    if (!resolve_options(options, &o)) return GREM_ERR_ARG;
    hipStream_t s = (hipStream_t)stream;
    if (k <= 255)
        return run_partition<RowT, uint8_t>(rowptr, colidx, n, k, slack, chunk, R, seed, labels_out,
                                            sizes_out, estimates_out, o, s);
    return run_partition<RowT, uint16_t>(rowptr, colidx, n, k, slack, chunk, R, seed, labels_out,
                                         sizes_out, estimates_out, o, s);
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

// A plan: the re-laid-out copy and the memory it lives in.
struct grem_plan {
    PlanData data;
    Arena mem;          // persistent allocations
};

extern "C" {

int64_t grem_capacity(int64_t n, int32_t k, double balance_slack) {
    if (n < 1 || k < 1 || !(balance_slack >= 1.0)) return -1;
    const int64_t even = (n + k - 1) / k;
    const double scaled = (double)n * balance_slack;
    const double per = scaled / (double)k;
    const int64_t widened = (int64_t)std::ceil(per);
    return even > widened ? even : widened;
}

size_t grem_workspace_bytes(int64_t n, int32_t k, int64_t chunk) {
    if (n < 1 || n > (int64_t)INT32_MAX || k < 1 || k > GREM_MAX_K || chunk < 1) return 0;
    return plain_bytes(n, k, chunk < n ? chunk : n, false);
}

size_t grem_workspace_bytes_two_phase(int64_t n, int64_t nnz, int32_t k, int64_t chunk, const grem_options *options) {
    if (n < 1 || n > (int64_t)INT32_MAX || nnz < 0 || k < 1 || k > GREM_MAX_K || chunk < 1) return 0;
    Opts o;
    if (!resolve_options(options, &o)) return 0;
    const int64_t cl = chunk < n ? chunk : n;
    const size_t plain = plain_bytes(n, k, cl, false);
    const TpGeom geo = tp_geometry(n, cl, o.col_bits, k);
    if (k > kSweepMaxK || !geo.ok) return plain;
    PlanDims d{};
    d.n = n;
    d.nnz = nnz;
    d.geo = geo;
    d.G = (size_t)geo.nch * (size_t)geo.nsl;
    d.hubs = (size_t)(nnz / o.hub_degree);                   // a hub has at least hub_degree entries
    if (d.hubs > (size_t)n) d.hubs = (size_t)n;
    d.npr = kMaxParts;
    d.nps = kMaxParts;
    {   // a chunk has at most one hub share per 64 * nblk hub entries (and at least one per 1024 hubs), never
        // more than slices
        size_t shares = (size_t)nnz / (64 * (size_t)geo.nblk) + d.hubs / 1024 + 1;
        if (shares > (size_t)geo.nsl) shares = (size_t)geo.nsl;
        d.nr = geo.nsl + (int)shares;
    }
    d.slots = plan_slots(nnz, geo, d.nr);
    SweepPlan pl{};
    TpTables tb{};
    u64 *pm = nullptr;
    uint32_t *T = nullptr;
    uint16_t *R = nullptr;
    CallState<uint8_t> st;
    TpState t;
    size_t total = carve_size([&](Carver &c) { state_common(c, st, n, cl, k); });
    total += carve_size([&](Carver &c) { plan_stage1(c, d, pl, pm); });
    total += carve_size([&](Carver &c) { plan_stage2(c, d, pl); });
    total += carve_size([&](Carver &c) { plan_stage3(c, d, tb, T, R); });
    // the intermediate copy and the per-call state take turns in one region; the state is largest for a
    // seeded run whose estimates need 32 bits
    const size_t temp = align_up((size_t)nnz * 4 + 16) + align_up((size_t)geo.nch * (size_t)d.nr * (size_t)geo.nblk * 4);
    const size_t chunk_hubs = d.hubs < (size_t)cl ? d.hubs : (size_t)cl;
    const size_t s16 = carve_size([&](Carver &c) { state_two_phase(c, t, n, k, d.slots, chunk_hubs, d.hubs, true, true, false, true); });
    const size_t s32 = carve_size([&](Carver &c) { state_two_phase(c, t, n, k, d.slots, chunk_hubs, d.hubs, true, false, false, true); });
    size_t tail = temp;
    if (s16 > tail) tail = s16;
    if (s32 > tail) tail = s32;
    total += tail;
    return total > plain ? total : plain;
}

int grem_set_workspace(void *dev_ptr, size_t bytes) {
    std::lock_guard<std::mutex> lock(g.mu);
    if ((dev_ptr == nullptr) != (bytes == 0)) return GREM_ERR_ARG;
    if (((uintptr_t)dev_ptr & 255u) != 0) return GREM_ERR_ARG;
    g.ws = dev_ptr;
    g.ws_bytes = bytes;
    return GREM_OK;
}

int grem_partition(const int64_t *rowptr, const int32_t *colidx, int64_t n, int32_t k,
                   double balance_slack, int64_t chunk, int32_t refine_passes, int32_t *labels_out,
                   void *stream) {
    return dispatch_labels<int64_t>(rowptr, colidx, n, k, balance_slack, chunk, refine_passes, nullptr,
                                    labels_out, nullptr, nullptr, nullptr, stream);
}

int grem_partition_seeded(const int64_t *rowptr, const int32_t *colidx, int64_t n, int32_t k,
                          double balance_slack, int64_t chunk, int32_t refine_passes,
                          const int32_t *seed_labels, int32_t *labels_out, void *stream) {
    return dispatch_labels<int64_t>(rowptr, colidx, n, k, balance_slack, chunk, refine_passes,
                                    seed_labels, labels_out, nullptr, nullptr, nullptr, stream);
}

int grem_partition_r32(const int32_t *rowptr, const int32_t *colidx, int64_t n, int32_t k,
                       double balance_slack, int64_t chunk, int32_t refine_passes, int32_t *labels_out,
                       void *stream) {
    return dispatch_labels<int32_t>(rowptr, colidx, n, k, balance_slack, chunk, refine_passes, nullptr,
                                    labels_out, nullptr, nullptr, nullptr, stream);
}

int grem_partition_seeded_r32(const int32_t *rowptr, const int32_t *colidx, int64_t n, int32_t k,
                              double balance_slack, int64_t chunk, int32_t refine_passes,
                              const int32_t *seed_labels, int32_t *labels_out, void *stream) {
    return dispatch_labels<int32_t>(rowptr, colidx, n, k, balance_slack, chunk, refine_passes,
                                    seed_labels, labels_out, nullptr, nullptr, nullptr, stream);
}

int grem_partition_opt(const void *rowptr, int32_t rowptr_bits, const int32_t *colidx, int64_t n,
                       int32_t k, double balance_slack, int64_t chunk, int32_t refine_passes,
                       const int32_t *seed_labels, int32_t *labels_out, int64_t *sizes_out,
                       uint32_t *estimates_out, const grem_options *options, void *stream) {
    if (rowptr_bits == 64)
        return dispatch_labels<int64_t>((const int64_t *)rowptr, colidx, n, k, balance_slack, chunk,
                                        refine_passes, seed_labels, labels_out, sizes_out,
                                        estimates_out, options, stream);
    if (rowptr_bits == 32)
        return dispatch_labels<int32_t>((const int32_t *)rowptr, colidx, n, k, balance_slack, chunk,
                                        refine_passes, seed_labels, labels_out, sizes_out,
                                        estimates_out, options, stream);
    return GREM_ERR_ARG;
}

int grem_partition_state(const void *rowptr, int32_t rowptr_bits, const int32_t *colidx, int64_t n,
                         int32_t k, double balance_slack, int64_t chunk, int32_t refine_passes,
                         const int32_t *seed_labels, int32_t *labels_out, int64_t *sizes_out,
                         uint32_t *estimates_out, void *stream) {
    return grem_partition_opt(rowptr, rowptr_bits, colidx, n, k, balance_slack, chunk, refine_passes, seed_labels,
                              labels_out, sizes_out, estimates_out, nullptr, stream);
}

int grem_plan_create(const void *rowptr, int32_t rowptr_bits, const int32_t *colidx, int64_t n, int64_t chunk,
                     const grem_options *options, void *stream, grem_plan **plan_out) {
    if (!plan_out) return GREM_ERR_ARG;
    *plan_out = nullptr;
    if (!rowptr || !colidx || n < 1 || n > (int64_t)INT32_MAX || chunk < 1 || (rowptr_bits != 32 && rowptr_bits != 64))
        return GREM_ERR_ARG;
    Opts o;
    if (!resolve_options(options, &o)) return GREM_ERR_ARG;
    const int64_t cl = chunk < n ? chunk : n;
    if (!tp_geometry(n, cl, o.col_bits, o.plan_max_k).ok) return GREM_ERR_ARG;
    grem_plan *p = new (std::nothrow) grem_plan();
    if (!p) return GREM_ERR_NOMEM;
    hipStream_t s = (hipStream_t)stream;
    p->mem.persistent = true;
    Arena temp;
    temp.stream = s;
    Launcher L{s};
    {
        std::lock_guard<std::mutex> lock(g.mu);
        L.level = g.prof_level;
    }
    L.mark();
    int rc = rowptr_bits == 64
                 ? build_plan<int64_t>(p->data, (const int64_t *)rowptr, colidx, n, cl, 0, o, p->mem, temp, L, true)
                 : build_plan<int32_t>(p->data, (const int32_t *)rowptr, colidx, n, cl, 0, o, p->mem, temp, L, true);
    L.mark();
    temp.release_all();
    if (hipStreamSynchronize(s) != hipSuccess && rc == GREM_OK) rc = GREM_ERR_HIP;
    if (rc != GREM_OK) {
        p->mem.release_all();
        delete p;
        return rc;
    }
    *plan_out = p;
    return GREM_OK;
}

int grem_plan_destroy(grem_plan *plan) {
    if (!plan) return GREM_OK;
    const int rc = hipDeviceSynchronize() == hipSuccess ? GREM_OK : GREM_ERR_HIP;
    plan->mem.release_all();
    delete plan;
    return rc;
}

size_t grem_plan_device_bytes(const grem_plan *plan) { return plan ? plan->mem.total : 0; }

int32_t grem_plan_max_k(const grem_plan *plan) { return plan ? plan->data.max_k : 0; }

size_t grem_plan_call_bytes(const grem_plan *plan, int32_t k, int32_t refine_passes, int32_t seeded,
                            int32_t with_estimates_out) {
    if (!plan || !plan->data.T || k < 1 || k > plan->data.max_k || refine_passes < 0 || refine_passes >= 32) return 0;
    const PlanData &P = plan->data;
    const bool use16 = (((unsigned long long)(P.hub_degree - 1)) << refine_passes) <= 65535ull;
    CallState<uint8_t> st;
    TpState t;
    return carve_size([&](Carver &c) { state_common(c, st, P.n, (int64_t)P.geo.chunk, k); }) +
           carve_size([&](Carver &c) {
               state_two_phase(c, t, P.n, k, P.slots, (size_t)P.max_chunk_hubs, (size_t)P.total_hubs, seeded != 0, use16,
                               with_estimates_out != 0, admission_takes_hubs(P, use16, with_estimates_out != 0));
           });
}

int grem_partition_planned(const grem_plan *plan, int32_t k, double balance_slack, int32_t refine_passes,
                           const int32_t *seed_labels, int32_t *labels_out, int64_t *sizes_out,
                           uint32_t *estimates_out, void *stream) {
    if (!plan || !plan->data.T || !labels_out || k < 1 || k > plan->data.max_k || refine_passes < 0 ||
        !(balance_slack >= 1.0) || std::isinf(balance_slack))
        return GREM_ERR_ARG;
    hipStream_t s = (hipStream_t)stream;
    Arena mem;
    mem.stream = s;
    Launcher L{s};
    {
        std::lock_guard<std::mutex> lock(g.mu);
        mem.base = (char *)g.ws;
        mem.cap = g.ws_bytes;
        L.level = g.prof_level;
    }
    L.mark();
    const int rc = plan->data.rowptr_bits == 64
                       ? run_two_phase<int64_t>(plan->data, k, balance_slack, refine_passes, seed_labels, labels_out,
                                                sizes_out, estimates_out, mem, L, nullptr)
                       : run_two_phase<int32_t>(plan->data, k, balance_slack, refine_passes, seed_labels, labels_out,
                                                sizes_out, estimates_out, mem, L, nullptr);
    mem.release_all();
    return rc;
}

int64_t grem_plan_n(const grem_plan *plan) { return plan ? plan->data.n : 0; }

namespace {

// cnt_nbrs of every vertex under a labelling that stays as it is, on a plan; `mem` supplies the
// run's state (the caller releases it)
int plan_counts(const grem_plan *plan, int32_t k, const int32_t *labels, uint32_t *counts_out, Arena &mem, Launcher &L) {
    // capacity n: whatever the labelling, no partition is over it
    return plan->data.rowptr_bits == 64
               ? run_two_phase<int64_t>(plan->data, k, (double)k, 0, labels, nullptr, nullptr, counts_out, mem, L, nullptr, true)
               : run_two_phase<int32_t>(plan->data, k, (double)k, 0, labels, nullptr, nullptr, counts_out, mem, L, nullptr, true);
}

void plan_call_setup(Arena &mem, Launcher &L, hipStream_t s) {
    mem.stream = s;
    std::lock_guard<std::mutex> lock(g.mu);
    mem.base = (char *)g.ws;
    mem.cap = g.ws_bytes;
    L.level = g.prof_level;
}

}  // namespace

int grem_plan_neighbour_counts(const grem_plan *plan, int32_t k, const int32_t *labels, uint32_t *counts_out,
                               void *stream) {
    if (!plan || !plan->data.T || !labels || !counts_out || k < 1 || k > plan->data.max_k) return GREM_ERR_ARG;
    hipStream_t s = (hipStream_t)stream;
    Arena mem;
    Launcher L{s};
    plan_call_setup(mem, L, s);
    L.mark();
    const int rc = plan_counts(plan, k, labels, counts_out, mem, L);
    mem.release_all();
    return rc;
}

int grem_plan_edge_cut(const grem_plan *plan, int32_t k, const int32_t *labels, int64_t *cut_entries_out,
                       void *stream) {
    if (!plan || !plan->data.T || !labels || !cut_entries_out || k < 1 || k > plan->data.max_k) return GREM_ERR_ARG;
    hipStream_t s = (hipStream_t)stream;
    Arena mem;
    Launcher L{s};
    plan_call_setup(mem, L, s);
    L.mark();
    const int64_t n = plan->data.n;
    uint32_t *counts = nullptr;
    if (!carve(mem, [&](Carver &c) { c.take(counts, (size_t)n * (size_t)k); })) return GREM_ERR_NOMEM;
    int rc = plan_counts(plan, k, labels, counts, mem, L);
    if (rc == GREM_OK) {
        int64_t blocks = (n + 255) / 256;
        if (blocks > 256 * 32) blocks = 256 * 32;
        L.run(GREM_KERNEL_EXPAND, [&] {
            hipLaunchKernelGGL(k_zero_u64, dim3(1), dim3(64), 0, s, (unsigned long long *)cut_entries_out, 1);
        });
        L.run(GREM_KERNEL_EXPAND, [&] {
            if (plan->data.rowptr_bits == 64)
                hipLaunchKernelGGL(k_cut_from_counts<int64_t>, dim3((unsigned)blocks), dim3(256), 0, s,
                                   (const int64_t *)plan->data.rowptr, labels, (const uint32_t *)counts, n, (int)k,
                                   (unsigned long long *)cut_entries_out);
            else
                hipLaunchKernelGGL(k_cut_from_counts<int32_t>, dim3((unsigned)blocks), dim3(256), 0, s,
                                   (const int32_t *)plan->data.rowptr, labels, (const uint32_t *)counts, n, (int)k,
                                   (unsigned long long *)cut_entries_out);
        });
        rc = L.err;
    }
    mem.release_all();
    return rc;
}

int grem_edge_cut(const int64_t *rowptr, const int32_t *colidx, int64_t n, const int32_t *labels,
                  int64_t *cut_entries_out, void *stream) {
    return run_edge_cut<int64_t>(rowptr, colidx, n, labels, cut_entries_out, stream);
}

int grem_edge_cut_r32(const int32_t *rowptr, const int32_t *colidx, int64_t n, const int32_t *labels,
                      int64_t *cut_entries_out, void *stream) {
    return run_edge_cut<int32_t>(rowptr, colidx, n, labels, cut_entries_out, stream);
}

int grem_profile_enable(int32_t level) {
    if (level < 0 || level > 2) return GREM_ERR_ARG;
    std::lock_guard<std::mutex> lock(g.mu);
    g.prof_level = level;
    return GREM_OK;
}

int grem_profile_reset(void) {
    std::lock_guard<std::mutex> lock(g.mu);
    for (auto &e : g.events) { g.pool.push_back(e.a); g.pool.push_back(e.b); }
    for (auto &e : g.marks) g.pool.push_back(e);
    g.events.clear();
    g.marks.clear();
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

int grem_profile_read_marks(double *ms_out, int32_t capacity) {
    if (!ms_out || capacity < 0) return GREM_ERR_ARG;
    std::lock_guard<std::mutex> lock(g.mu);
    int written = 0;
    for (size_t i = 1; i < g.marks.size() && written < capacity; ++i) {
        if (hipEventSynchronize(g.marks[i]) != hipSuccess) return GREM_ERR_HIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g.marks[i - 1], g.marks[i]) != hipSuccess) return GREM_ERR_HIP;
        ms_out[written++] = ms;
    }
    return written;
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
