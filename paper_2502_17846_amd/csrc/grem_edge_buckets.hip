// Edge buckets for gfx950 (Armada paper, Sec. 3, storage layer): given the partition of every node, the
// edges are grouped so that bucket (i, j) holds the edges from nodes of partition i to nodes of
// partition j, each bucket stored as one sequential list; buckets follow each other in the order of
// i*k + j and an edge keeps its stream position relative to the other edges of its bucket (the paper
// fixes no order inside a bucket; this makes the result unique).
//
// A stable counting sort by key = label[src]*k + label[dst], one workgroup per tile of the stream:
//   k_eb_hist     keys of the tile's edges (two look-ups into a byte-per-node label table), stored as
//                 uint16 for the second pass, and the tile's histogram over the k*k buckets in LDS
//                 -> H[tile][bucket]
//   k_eb_colsum / k_eb_bases / k_eb_colscan
//                 exclusive prefix sums of H in bucket-major order (bucket, then tile): H[tile][bucket]
//                 becomes the output position of the tile's first edge of that bucket
//   k_eb_scatter  the tile again, 256 edges at a time in stream order: lanes with equal keys are matched
//                 inside a wave (one ballot per key bit), the waves take their ranges from the LDS
//                 cursors one after the other, every edge is written to cursor + rank
//   k_eb_scatter_lds  (tiles of 4,096 edges, up to 1,024 buckets) the tile is sorted in LDS first and then
//                 written out run by run
#include <hip/hip_runtime.h>

#include <cstdint>

#include "grem.h"

namespace {

typedef unsigned long long u64;
constexpr int kEbBlock = 256;
constexpr int kEbWaves = kEbBlock / 64;
constexpr int kEbMaxK = 128;                       // k*k*4 bytes of LDS: 64 KB at k = 128
constexpr int64_t kEbMaxCells = (int64_t)1 << 27;  // tiles * k*k
constexpr int64_t kEbMinTile = 4096;
constexpr uint32_t kBadLabel = 0xFFu;

__global__ __launch_bounds__(256) void k_eb_zero(uint32_t* p, size_t count)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) p[i] = 0u;
}

// one byte per node; labels outside [0, k) become kBadLabel
__global__ __launch_bounds__(256) void k_eb_compact(int64_t n, const int32_t* __restrict__ labels, int32_t k, uint8_t* L8)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += stride) {
        const int32_t l = labels[v];
        L8[v] = (l >= 0 && l < k) ? (uint8_t)l : (uint8_t)kBadLabel;
    }
}

// flags[0]: an endpoint outside [0, n); flags[1]: an endpoint whose label lies outside [0, k)
__global__ __launch_bounds__(kEbBlock) void k_eb_hist(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                                      int64_t m, uint32_t n, int64_t tile, const uint8_t* __restrict__ L8,
                                                      int32_t k, uint16_t* __restrict__ key16, uint32_t* __restrict__ H,
                                                      uint32_t* flags)
{
    extern __shared__ uint32_t hist[];
    const int k2 = k * k;
    for (int b = threadIdx.x; b < k2; b += kEbBlock) hist[b] = 0u;
    __syncthreads();
    const int64_t lo = (int64_t)blockIdx.x * tile, hi = lo + tile < m ? lo + tile : m;
    bool bad = false, outside = false;
    for (int64_t e = lo + threadIdx.x; e < hi; e += kEbBlock) {
        const uint32_t s = (uint32_t)src[e], d = (uint32_t)dst[e];
        uint32_t key = 0u;
        if (s < n && d < n) {
            const uint32_t ls = L8[s], ld = L8[d];
            if (ls < (uint32_t)k && ld < (uint32_t)k) key = ls * (uint32_t)k + ld;
            else bad = true;
        } else {
            outside = true;
        }
        key16[e] = (uint16_t)key;
        atomicAdd(&hist[key], 1u);
    }
    if (outside) flags[0] = 1u;
    if (bad) flags[1] = 1u;
    __syncthreads();
    uint32_t* row = H + (size_t)blockIdx.x * (size_t)k2;
    for (int b = threadIdx.x; b < k2; b += kEbBlock) row[b] = hist[b];
}

// partial[b*S + seg] = sum over the tiles of segment seg of H[tile][b]
__global__ __launch_bounds__(256) void k_eb_colsum(const uint32_t* __restrict__ H, int64_t tiles, int32_t k2, int32_t S,
                                                   int64_t seg_len, uint32_t* partial)
{
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (int64_t)k2 * S) return;
    const int b = (int)(id % k2), seg = (int)(id / k2);
    const int64_t t0 = seg * seg_len, t1 = t0 + seg_len < tiles ? t0 + seg_len : tiles;
    uint32_t sum = 0;
    for (int64_t t = t0; t < t1; ++t) sum += H[(size_t)t * k2 + b];
    partial[(size_t)b * S + seg] = sum;
}

// One workgroup: exclusive prefix sums of partial (bucket-major) in place, and the buckets' offsets.
__global__ __launch_bounds__(1024) void k_eb_bases(uint32_t* partial, int64_t len, int32_t k2, int32_t S,
                                                   int64_t m, int64_t* bucket_offsets)
{
    __shared__ uint32_t wsum[16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t carry = 0;
    for (int64_t base = 0; base < len; base += 1024) {
        const int64_t i = base + threadIdx.x;
        const uint32_t x = i < len ? partial[i] : 0u;
        uint32_t incl = x;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t y = __shfl_up(incl, o);
            if (lane >= o) incl += y;
        }
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        uint32_t before = 0, all = 0;
        for (int q = 0; q < 16; ++q) {
            const uint32_t t = wsum[q];
            if (q < wave) before += t;
            all += t;
        }
        if (i < len) {
            const uint32_t excl = carry + before + incl - x;
            partial[i] = excl;
            if (i % S == 0) bucket_offsets[i / S] = (int64_t)excl;
        }
        carry += all;
        __syncthreads();
    }
    if (threadIdx.x == 0) bucket_offsets[k2] = m;
}

// H[tile][b] becomes the output position of the tile's first edge of bucket b
__global__ __launch_bounds__(256) void k_eb_colscan(uint32_t* __restrict__ H, int64_t tiles, int32_t k2, int32_t S,
                                                    int64_t seg_len, const uint32_t* __restrict__ segbase)
{
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (int64_t)k2 * S) return;
    const int b = (int)(id % k2), seg = (int)(id / k2);
    const int64_t t0 = seg * seg_len, t1 = t0 + seg_len < tiles ? t0 + seg_len : tiles;
    uint32_t run = segbase[(size_t)b * S + seg];
    for (int64_t t = t0; t < t1; ++t) {
        const uint32_t c = H[(size_t)t * k2 + b];
        H[(size_t)t * k2 + b] = run;
        run += c;
    }
}

__global__ __launch_bounds__(kEbBlock) void k_eb_scatter(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                                         int64_t m, int64_t tile, const uint16_t* __restrict__ key16,
                                                         int32_t k2, int32_t key_bits, const uint32_t* __restrict__ H,
                                                         int32_t* __restrict__ out_src, int32_t* __restrict__ out_dst)
{
    extern __shared__ uint32_t cur[];
    const uint32_t* row = H + (size_t)blockIdx.x * (size_t)k2;
    for (int b = threadIdx.x; b < k2; b += kEbBlock) cur[b] = row[b];
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const u64 below = (1ull << lane) - 1ull;
    const int64_t lo = (int64_t)blockIdx.x * tile, hi = lo + tile < m ? lo + tile : m;
    for (int64_t base = lo; base < hi; base += kEbBlock) {        // uniform trip count over the workgroup
        const int64_t e = base + threadIdx.x;
        const bool valid = e < hi;
        uint32_t key = 0u;
        int32_t s = 0, d = 0;
        if (valid) { key = key16[e]; s = src[e]; d = dst[e]; }
        // lanes of this wave that hold the same key
        u64 same = __ballot(valid);
        for (int bit = 0; bit < key_bits; ++bit) {
            const bool one = (key >> bit) & 1u;
            const u64 b = __ballot(one);
            same &= one ? b : ~b;
        }
        const uint32_t rank = __popcll(same & below);
        uint32_t first = 0u;
        for (int w = 0; w < kEbWaves; ++w) {
            if (wave == w && valid && rank == 0u) {
                first = cur[key];
                cur[key] = first + (uint32_t)__popcll(same);
            }
            __syncthreads();
        }
        const int leader = valid ? __builtin_ctzll(same) : lane;
        const uint32_t pos = __shfl(first, leader) + rank;
        if (valid) { out_src[pos] = s; out_dst[pos] = d; }
    }
}

// The same placement for tiles of kEbMinTile edges and at most kEbLdsBuckets buckets, with the tile sorted
// in LDS first so that the output is written in whole runs: each of the four waves owns a quarter of the
// tile (consecutive stream positions), counts it, the counts become per-wave cursors into the tile's sorted
// order (bucket, then wave, then stream position = stable), every wave places its edges into LDS without
// waiting for the others, and the sorted tile is written out with consecutive lanes on consecutive
// addresses of a bucket's run.
constexpr int kEbLdsBuckets = 1024;
constexpr int kEbSeg = (int)(kEbMinTile / kEbWaves);

__global__ __launch_bounds__(kEbBlock) void k_eb_scatter_lds(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                                             int64_t m, const uint16_t* __restrict__ key16, int32_t k2,
                                                             int32_t key_bits, const uint32_t* __restrict__ H,
                                                             int32_t* __restrict__ out_src, int32_t* __restrict__ out_dst)
{
    extern __shared__ uint32_t lds[];
    int32_t* ssrc = (int32_t*)lds;                          // kEbMinTile
    int32_t* sdst = ssrc + kEbMinTile;                      // kEbMinTile
    uint32_t* gstart = (uint32_t*)(sdst + kEbMinTile);      // k2: output position of the tile's first edge of a bucket
    uint32_t* lstart = gstart + k2;                         // k2: the same inside the sorted tile
    uint32_t* curw = lstart + k2;                           // kEbWaves * k2: counts, then cursors, per wave
    uint16_t* skey = (uint16_t*)(curw + kEbWaves * k2);     // kEbMinTile
    __shared__ uint32_t tsum[kEbBlock];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t lo = (int64_t)blockIdx.x * kEbMinTile, hi = lo + kEbMinTile < m ? lo + kEbMinTile : m;
    const int count = (int)(hi - lo);
    const uint32_t* row = H + (size_t)blockIdx.x * (size_t)k2;
    for (int b = threadIdx.x; b < k2; b += kEbBlock) gstart[b] = row[b];
    for (int b = threadIdx.x; b < kEbWaves * k2; b += kEbBlock) curw[b] = 0u;
    __syncthreads();
    // counts of the wave's quarter
    const int seg0 = wave * kEbSeg, seg1 = seg0 + kEbSeg < count ? seg0 + kEbSeg : count;
    uint32_t* mine = curw + wave * k2;
    for (int p = seg0 + lane; p < seg1; p += 64) atomicAdd(&mine[key16[lo + p]], 1u);
    __syncthreads();
    // exclusive sums over (bucket, wave): a thread owns k2 / kEbBlock consecutive buckets (at least one)
    const int per = (k2 + kEbBlock - 1) / kEbBlock;
    const int b0 = threadIdx.x * per, b1 = b0 + per < k2 ? b0 + per : k2;
    uint32_t own = 0;
    for (int b = b0; b < b1; ++b)
        for (int w = 0; w < kEbWaves; ++w) own += curw[w * k2 + b];
    tsum[threadIdx.x] = own;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int t = 0; t < kEbBlock; ++t) { const uint32_t v = tsum[t]; tsum[t] = run; run += v; }
    }
    __syncthreads();
    uint32_t run = tsum[threadIdx.x];
    for (int b = b0; b < b1; ++b) {
        lstart[b] = run;
        for (int w = 0; w < kEbWaves; ++w) { const uint32_t c = curw[w * k2 + b]; curw[w * k2 + b] = run; run += c; }
    }
    __syncthreads();
    // every wave places its quarter, 64 edges at a time in stream order
    const u64 below = (1ull << lane) - 1ull;
    for (int base = seg0; base < seg1; base += 64) {
        const int p = base + lane;
        const bool valid = p < seg1;
        uint32_t key = 0u;
        int32_t s = 0, d = 0;
        if (valid) { key = key16[lo + p]; s = src[lo + p]; d = dst[lo + p]; }
        u64 same = __ballot(valid);
        for (int bit = 0; bit < key_bits; ++bit) {
            const bool one = (key >> bit) & 1u;
            const u64 b = __ballot(one);
            same &= one ? b : ~b;
        }
        const uint32_t rank = __popcll(same & below);
        uint32_t first = 0u;
        if (valid && rank == 0u) { first = mine[key]; mine[key] = first + (uint32_t)__popcll(same); }
        const int leader = valid ? __builtin_ctzll(same) : lane;
        const uint32_t pos = __shfl(first, leader) + rank;
        if (valid) { ssrc[pos] = s; sdst[pos] = d; skey[pos] = (uint16_t)key; }
    }
    __syncthreads();
    for (int p = threadIdx.x; p < count; p += kEbBlock) {
        const uint32_t key = skey[p];
        const uint32_t at = gstart[key] + ((uint32_t)p - lstart[key]);
        out_src[at] = ssrc[p];
        out_dst[at] = sdst[p];
    }
}

inline size_t eb_align(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

extern "C" int grem_edge_buckets(const int32_t* src, const int32_t* dst, int64_t m, int64_t n,
                                 const int32_t* labels, int32_t k, int32_t* out_src, int32_t* out_dst,
                                 int64_t* bucket_offsets, void* stream_)
{
    if (!src || !dst || !labels || !out_src || !out_dst || !bucket_offsets || m < 1 || m > (int64_t)0xFFFFFFFFll ||
        n < 1 || n > INT32_MAX || k < 1 || k > kEbMaxK)
        return GREM_ERR_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    const int32_t k2 = k * k;
    int64_t tile = (m * k2 + kEbMaxCells - 1) / kEbMaxCells;
    if (tile < kEbMinTile) tile = kEbMinTile;
    tile = (tile + kEbBlock - 1) / kEbBlock * kEbBlock;
    const int64_t tiles = (m + tile - 1) / tile;
    int32_t S = 65536 / k2;
    if (S < 1) S = 1;
    if (S > tiles) S = (int32_t)tiles;
    const int64_t seg_len = (tiles + S - 1) / S;
    int key_bits = 0;
    while ((1 << key_bits) < k2) ++key_bits;

    size_t off = 0;
    auto carve = [&](size_t bytes) { const size_t at = off; off += eb_align(bytes); return at; };
    const size_t o_flags = carve(256), o_l8 = carve((size_t)n), o_key = carve((size_t)m * 2);
    const size_t o_h = carve((size_t)tiles * k2 * 4), o_part = carve((size_t)k2 * S * 4);
    uint8_t* ws = nullptr;
    if (hipMallocAsync((void**)&ws, off, stream) != hipSuccess) { (void)hipGetLastError(); return GREM_ERR_NOMEM; }
    auto fail = [&](int code) { (void)hipGetLastError(); (void)hipStreamSynchronize(stream); (void)hipFreeAsync(ws, stream); return code; };
    uint32_t* flags = (uint32_t*)(ws + o_flags);
    uint8_t* L8 = ws + o_l8;
    uint16_t* key16 = (uint16_t*)(ws + o_key);
    uint32_t* H = (uint32_t*)(ws + o_h);
    uint32_t* partial = (uint32_t*)(ws + o_part);
    const size_t lds = (size_t)k2 * 4;
    if (lds > 48 * 1024) {
        if (hipFuncSetAttribute((const void*)k_eb_hist, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess ||
            hipFuncSetAttribute((const void*)k_eb_scatter, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return fail(GREM_ERR_HIP);
    }
    auto grid = [](int64_t items, int64_t cap) { int64_t g = (items + 255) / 256; if (g < 1) g = 1; if (g > cap) g = cap; return (int)g; };
    hipLaunchKernelGGL(k_eb_zero, dim3(1), dim3(256), 0, stream, flags, (size_t)64);
    uint32_t host_flags[2] = {0, 0};
    hipLaunchKernelGGL(k_eb_compact, dim3(grid(n, 16384)), dim3(256), 0, stream, n, labels, k, L8);
    hipLaunchKernelGGL(k_eb_hist, dim3((unsigned)tiles), dim3(kEbBlock), lds, stream, src, dst, m, (uint32_t)n, tile, L8, k, key16, H, flags);
    if (hipMemcpyAsync(host_flags, flags, sizeof(host_flags), hipMemcpyDeviceToHost, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess)
        return fail(GREM_ERR_HIP);
    if (host_flags[0] || host_flags[1]) return fail(GREM_ERR_ARG);
    const int64_t cells = (int64_t)k2 * S;
    hipLaunchKernelGGL(k_eb_colsum, dim3(grid(cells, 1 << 20)), dim3(256), 0, stream, H, tiles, k2, S, seg_len, partial);
    hipLaunchKernelGGL(k_eb_bases, dim3(1), dim3(1024), 0, stream, partial, cells, k2, S, m, bucket_offsets);
    hipLaunchKernelGGL(k_eb_colscan, dim3(grid(cells, 1 << 20)), dim3(256), 0, stream, H, tiles, k2, S, seg_len, partial);
    if (tile == kEbMinTile && k2 <= kEbLdsBuckets) {
        const size_t lds2 = (size_t)kEbMinTile * 10 + (size_t)k2 * 4 * (2 + kEbWaves);
        if (hipFuncSetAttribute((const void*)k_eb_scatter_lds, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2) != hipSuccess)
            return fail(GREM_ERR_HIP);
        hipLaunchKernelGGL(k_eb_scatter_lds, dim3((unsigned)tiles), dim3(kEbBlock), lds2, stream, src, dst, m, key16, k2, key_bits, H,
                           out_src, out_dst);
    } else {
        hipLaunchKernelGGL(k_eb_scatter, dim3((unsigned)tiles), dim3(kEbBlock), lds, stream, src, dst, m, tile, key16, k2, key_bits, H,
                           out_src, out_dst);
    }
    int rc = hipGetLastError() == hipSuccess ? GREM_OK : GREM_ERR_HIP;
    if (hipFreeAsync(ws, stream) != hipSuccess) rc = GREM_ERR_HIP;
    return rc;
}
