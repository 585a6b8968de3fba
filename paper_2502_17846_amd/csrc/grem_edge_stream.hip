// GREM over a stream of edge chunks, two partitions, for gfx950 (Armada paper, Sec. 4.1, Alg. 1
// "GREM Bipartite Graph Partitioning" with the helpers of Alg. 2, in the stream model the paper
// states them in: an edge list in random order, a chunk is c_size consecutive edges, the chunk's
// nodes are the distinct endpoints of its edges and each is (re)evaluated from the chunk's edges).
//
// Chunk-synchronous form: every decision of a chunk reads labels and sizes as of the chunk's start;
// moves are admitted in ascending node id while the target has room; rejected refined nodes stay;
// rejected new nodes are placed one by one, ascending id, in the currently smaller partition.
//
// Data layout (device memory)
//   Lb    uint8[n]      label 0/1, 0xFF = unassigned (one byte per random look-up)
//   hc    uint64[n]     fresh counts of the current chunk: low half = neighbours in partition 0, high
//                       half = neighbours in partition 1; one 64-bit atomic per edge end.  All zero
//                       between chunks (the scoring kernel clears what it reads).
//   est   double[n][2]  Alg. 1's nbr_counts
//   mark  uint64[n/64]  bit v set = v is an endpoint of a chunk edge whose other end has no label.
//                       A node belongs to the current chunk iff hc[v] != 0 or its bit is set.
//                       Bitmaps are ordered sets: bit order is id order, so ranks by id are prefix
//                       pop-counts.
//   mv0, mv1, ov        bitmaps of the same shape: nodes asking to move to partition 0 / 1, and new
//                       nodes whose request was rejected
// Per chunk: k_es_count (the edges: two label look-ups, bitmap marks and count atomics per edge) ->
// k_es_score (one lane per node, a wave walking over its 64 bitmap words: blend, assign, mover
// ballots) -> a one-workgroup scan of the per-workgroup mover counts -> k_es_apply (ranks = scanned
// offset + pop-count prefix; admitted moves relabel) -> a one-workgroup scan (overflow ranks, size
// deltas, closed-form sizes after the spill) -> k_es_spill (closed-form target of the j-th rejected
// node).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>
#include <vector>

#include "grem.h"

namespace {

constexpr int kBlock = 1024;                 // per-node kernels: 16 waves
constexpr int kWordsPerBlock = kBlock / 64;   // waves per workgroup
constexpr int kWaveWords = 64;               // bitmap words a wave of the per-node kernels owns
constexpr uint32_t kNone = 0xFFu;
constexpr int kCountBlock = 256;
constexpr int kCountUnroll = 4;              // edges in flight per thread of k_es_count

typedef unsigned long long u64;

__global__ __launch_bounds__(256) void k_es_fill64(u64* p, size_t count, u64 value)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) p[i] = value;
}

// flags[0] = 1 if any endpoint lies outside [0, n)
__global__ __launch_bounds__(256) void k_es_check(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                                  int64_t m, uint32_t n, uint32_t* flags)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    bool bad = false;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < m; e += stride)
        bad |= ((uint32_t)src[e] >= n) | ((uint32_t)dst[e] >= n);
    if (bad) flags[0] = 1u;
}

// c_nodes of a chunk as a bitmap (Alg. 1: unique_nodes_in_edges)
__global__ __launch_bounds__(kCountBlock) void k_es_mark(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                                         int64_t lo, int64_t hi, u64* mark)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = lo + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < hi; e += stride) {
        const uint32_t s = (uint32_t)src[e], d = (uint32_t)dst[e];
        atomicOr(&mark[s >> 6], 1ull << (s & 63u));
        atomicOr(&mark[d >> 6], 1ull << (d & 63u));
    }
}

// Alg. 1, first chunk: the chunk's nodes take seed_algo's labels; sizes are counted.
// flags[1] = 1 if a node of the chunk has a seed label other than 0 or 1.
__global__ __launch_bounds__(kBlock) void k_es_seed(int64_t words, const u64* __restrict__ mark,
                                                    const int32_t* __restrict__ seed, uint8_t* Lb,
                                                    u64* S, uint32_t* flags)
{
    __shared__ uint32_t c0[kWordsPerBlock], c1[kWordsPerBlock];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t w = (int64_t)blockIdx.x * kWordsPerBlock + wave;
    const u64 word = w < words ? mark[w] : 0ull;
    const bool on = (word >> lane) & 1ull;
    int s = -1;
    if (on) {
        const int64_t v = w * 64 + lane;
        s = seed[v];
        if (s == 0 || s == 1) Lb[v] = (uint8_t)s;
        else flags[1] = 1u;
    }
    const u64 b0 = __ballot(on && s == 0), b1 = __ballot(on && s == 1);
    if (lane == 0) { c0[wave] = __popcll(b0); c1[wave] = __popcll(b1); }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t a = 0, b = 0;
        for (int i = 0; i < kWordsPerBlock; ++i) { a += c0[i]; b += c1[i]; }
        if (a) atomicAdd(&S[0], (u64)a);
        if (b) atomicAdd(&S[1], (u64)b);
    }
}

// cnt_nbrs (Alg. 2) for every node of the chunk at once: each edge adds one to the count its two
// ends keep for the partition of the other end (a loop counts once, for the node itself).  An
// unassigned other end adds nothing; the node's bit in `mark` is set instead, so that a node of the
// chunk is known by a non-zero count or its bit: one atomic per edge end either way.
__global__ __launch_bounds__(kCountBlock) void k_es_count(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                                          int64_t lo, int64_t hi, const uint8_t* __restrict__ Lb,
                                                          u64* mark, u64* hc)
{
    const int64_t threads = (int64_t)gridDim.x * blockDim.x;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t base = lo + tid; base < hi; base += threads * kCountUnroll) {
        uint32_t s[kCountUnroll], d[kCountUnroll], ls[kCountUnroll], ld[kCountUnroll];
        bool in[kCountUnroll];
#pragma unroll
        for (int u = 0; u < kCountUnroll; ++u) {
            const int64_t e = base + (int64_t)u * threads;
            in[u] = e < hi;
            s[u] = in[u] ? (uint32_t)src[e] : 0u;
            d[u] = in[u] ? (uint32_t)dst[e] : 0u;
        }
#pragma unroll
        for (int u = 0; u < kCountUnroll; ++u) {
            ls[u] = in[u] ? (uint32_t)Lb[s[u]] : kNone;
            ld[u] = in[u] ? (uint32_t)Lb[d[u]] : kNone;
        }
#pragma unroll
        for (int u = 0; u < kCountUnroll; ++u) {
            if (!in[u]) continue;
            if (ld[u] != kNone) atomicAdd(&hc[s[u]], ld[u] ? (1ull << 32) : 1ull);
            else atomicOr(&mark[s[u] >> 6], 1ull << (s[u] & 63u));
            if (d[u] != s[u]) {
                if (ls[u] != kNone) atomicAdd(&hc[d[u]], ls[u] ? (1ull << 32) : 1ull);
                else atomicOr(&mark[d[u] >> 6], 1ull << (d[u] & 63u));
            }
        }
    }
}

// The two-partition choice of Alg. 2, on sizes from which the node itself has been taken out: the
// side that holds strictly more of the node's neighbours wins when it still has room; with no such
// side (equal estimates, or the richer side full) the smaller partition takes the node, 0 on a tie.
__device__ __forceinline__ int es_assign(double nbrs0, double nbrs1, long long s0, long long s1, long long P)
{
    const int lean = (nbrs1 > nbrs0) - (nbrs0 > nbrs1);   // +1: towards 1, -1: towards 0, 0: neither
    if (lean != 0) {
        const int p = lean > 0;
        if ((p ? s1 : s0) < P) return p;
    }
    return s1 < s0;
}

// value of x in lane i, i uniform over the wave
__device__ __forceinline__ u64 es_bcast(u64 x, int i)
{
    const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)x, i);
    const uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(x >> 32), i);
    return ((u64)hi << 32) | lo;
}

__device__ __forceinline__ uint32_t es_wave_sum(uint32_t x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// exclusive prefix sum over the lanes of a wave
__device__ __forceinline__ uint32_t es_wave_exclusive(uint32_t x, int lane)
{
    uint32_t incl = x;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t y = __shfl_up(incl, o);
        if (lane >= o) incl += y;
    }
    return incl - x;
}

// The per-node kernels: a wave owns kWaveWords = 64 consecutive bitmap words (lane i holds word i)
// and walks over them (k_es_score: all of them, reading the counts of their nodes; the others: those
// that have a bit set), one lane per node of the word; a workgroup of 16 waves owns 1024 words =
// 65536 nodes.
//
// k_es_score -- Alg. 1: blend the stored estimate with the fresh counts when the node has a label,
// store the estimate, ask `assign` for a partition.  Nodes that want to move are recorded in mv0 /
// mv1 (wave ballots), their numbers per workgroup in bs0 / bs1.  Clears what it consumed (hc, mark).
// first: the seeded first chunk (estimates only).  fixed: fixed greedy decisions (a node that has a
// label is left alone).
__global__ __launch_bounds__(kBlock) void k_es_score(int64_t n, int64_t words, int first, int fixed, long long P,
                                                     const u64* __restrict__ S, u64* mark, u64* hc,
                                                     const uint8_t* __restrict__ Lb, double2* est,
                                                     u64* mv0, u64* mv1, uint32_t* bs0, uint32_t* bs1)
{
    __shared__ uint32_t c0[kWordsPerBlock], c1[kWordsPerBlock];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t word0 = ((int64_t)blockIdx.x * kWordsPerBlock + wave) * kWaveWords;
    const bool mine = word0 + lane < words;
    const u64 myword = mine ? mark[word0 + lane] : 0ull;
    const long long S0 = (long long)S[0], S1 = (long long)S[1];
    const int count = words - word0 < kWaveWords ? (int)(words - word0) : kWaveWords;   // <= 0: nothing
    u64 out0 = 0ull, out1 = 0ull;
    int64_t v = word0 * 64 + lane;
    u64 hnext = (count > 0 && v < n) ? hc[v] : 0ull;
    for (int i = 0; i < count; ++i, v += 64) {
        const u64 h = hnext;
        hnext = (i + 1 < count && v + 64 < n) ? hc[v + 64] : 0ull;
        const u64 word = es_bcast(myword, i);
        int want = -1;
        if (h != 0ull || ((word >> lane) & 1ull)) {
            if (h) hc[v] = 0ull;
            const uint32_t old = Lb[v];
            double nbrs0 = (double)(uint32_t)h, nbrs1 = (double)(uint32_t)(h >> 32);
            if (first) {
                est[v] = make_double2(nbrs0, nbrs1);
            } else if (!(fixed && old != kNone)) {
                if (old != kNone) {
                    const double2 prev = est[v];
                    nbrs0 = (prev.x + nbrs0) * 0.5;
                    nbrs1 = (prev.y + nbrs1) * 0.5;
                }
                est[v] = make_double2(nbrs0, nbrs1);
                const int t = es_assign(nbrs0, nbrs1, S0 - (old == 0u), S1 - (old == 1u), P);
                if ((uint32_t)t != old) want = t;
            }
        }
        const u64 m0 = __ballot(want == 0), m1 = __ballot(want == 1);
        if (lane == i) { out0 = m0; out1 = m1; }
    }
    if (mine) {
        mv0[word0 + lane] = out0; mv1[word0 + lane] = out1;
        if (myword) mark[word0 + lane] = 0ull;
    }
    const uint32_t a = es_wave_sum(__popcll(out0)), b = es_wave_sum(__popcll(out1));
    if (lane == 0) { c0[wave] = a; c1[wave] = b; }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t x = 0, y = 0;
        for (int q = 0; q < kWordsPerBlock; ++q) { x += c0[q]; y += c1[q]; }
        bs0[blockIdx.x] = x; bs1[blockIdx.x] = y;
    }
}

// exclusive prefix sums of in[0..len) into out, by one workgroup of kBlock threads; returns the total
__device__ uint32_t es_block_scan(const uint32_t* __restrict__ in, uint32_t* __restrict__ out, int64_t len,
                                  uint32_t* wsum /* kWordsPerBlock words of LDS */)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t carry = 0;
    for (int64_t base = 0; base < len; base += kBlock) {
        const int64_t i = base + threadIdx.x;
        const uint32_t x = i < len ? in[i] : 0u;
        const uint32_t excl = es_wave_exclusive(x, lane);
        if (lane == 63) wsum[wave] = excl + x;
        __syncthreads();
        uint32_t before = 0, all = 0;
        for (int q = 0; q < kWordsPerBlock; ++q) {
            const uint32_t t = wsum[q];
            if (q < wave) before += t;
            all += t;
        }
        if (i < len) out[i] = carry + before + excl;
        carry += all;
        __syncthreads();
    }
    return carry;
}

__global__ __launch_bounds__(kBlock) void k_es_scan_movers(int64_t blocks, const uint32_t* bs0, const uint32_t* bs1,
                                                           uint32_t* bo0, uint32_t* bo1)
{
    __shared__ uint32_t wsum[kWordsPerBlock];
    (void)es_block_scan(bs0, bo0, blocks, wsum);
    (void)es_block_scan(bs1, bo1, blocks, wsum);
}

// Admission: a mover whose rank among the chunk's requests for its target (ascending id) is below
// the room the target had when the chunk started is relabelled (fix_sizes, Alg. 2, as per-workgroup
// deltas); a rejected node without a label is recorded in ov.  A wave that has movers copies the
// 4,096 labels of its 64 words into LDS with wide loads, every lane then walks the movers of its own
// word there, and the labels are written back if any changed (lb_bytes: the label array's allocated
// size, a multiple of 16).
__global__ __launch_bounds__(kBlock) void k_es_apply(int64_t words, long long P, const u64* __restrict__ S,
                                                     const u64* __restrict__ mv0, const u64* __restrict__ mv1,
                                                     const uint32_t* __restrict__ bo0, const uint32_t* __restrict__ bo1,
                                                     uint8_t* Lb, int64_t lb_bytes, u64* ov, uint32_t* bso, int32_t* bd0,
                                                     int32_t* bd1)
{
    extern __shared__ uint4 slab4[];                  // kBlock * 64 bytes: 4 KB per wave
    __shared__ uint32_t c0[kWordsPerBlock], c1[kWordsPerBlock], co[kWordsPerBlock];
    __shared__ int32_t d0[kWordsPerBlock], d1[kWordsPerBlock];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t word0 = ((int64_t)blockIdx.x * kWordsPerBlock + wave) * kWaveWords;
    const bool mine = word0 + lane < words;
    const u64 my0 = mine ? mv0[word0 + lane] : 0ull, my1 = mine ? mv1[word0 + lane] : 0ull;
    const uint32_t p0 = __popcll(my0), p1 = __popcll(my1);
    const uint32_t ex0 = es_wave_exclusive(p0, lane), ex1 = es_wave_exclusive(p1, lane);
    if (lane == 63) { c0[wave] = ex0 + p0; c1[wave] = ex1 + p1; }
    __syncthreads();
    uint32_t base0 = bo0[blockIdx.x], base1 = bo1[blockIdx.x];
    for (int q = 0; q < wave; ++q) { base0 += c0[q]; base1 += c1[q]; }
    const long long room0 = P - (long long)S[0], room1 = P - (long long)S[1];
    u64 outo = 0ull;
    int32_t delta0 = 0, delta1 = 0;
    const u64 movers = __ballot((my0 | my1) != 0ull);
    uint4* wslab4 = slab4 + wave * (kWaveWords * 64 / 16);
    const int64_t byte0 = word0 * 64;
    if (movers) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int q = u * 64 + lane;
            if (byte0 + (int64_t)(q + 1) * 16 <= lb_bytes) wslab4[q] = *reinterpret_cast<const uint4*>(Lb + byte0 + (int64_t)q * 16);
        }
    }
    // a lane walks the movers of its own word, in id order; ranks continue from the words before it
    uint8_t* mine64 = reinterpret_cast<uint8_t*>(wslab4) + lane * 64;
    bool dirty = false;
    long long r0 = (long long)base0 + ex0, r1 = (long long)base1 + ex1;
    for (u64 todo = my0; todo; todo &= todo - 1ull, ++r0) {
        const int b = __builtin_ctzll(todo);
        const uint32_t old = mine64[b];
        if (r0 < room0) { mine64[b] = 0; dirty = true; delta0 += 1; delta1 -= (int32_t)(old == 1u); }
        else if (old == kNone) outo |= 1ull << b;
    }
    for (u64 todo = my1; todo; todo &= todo - 1ull, ++r1) {
        const int b = __builtin_ctzll(todo);
        const uint32_t old = mine64[b];
        if (r1 < room1) { mine64[b] = 1; dirty = true; delta1 += 1; delta0 -= (int32_t)(old == 0u); }
        else if (old == kNone) outo |= 1ull << b;
    }
    delta0 = (int32_t)es_wave_sum((uint32_t)delta0);
    delta1 = (int32_t)es_wave_sum((uint32_t)delta1);
    if (__ballot(dirty)) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int q = u * 64 + lane;
            if (byte0 + (int64_t)(q + 1) * 16 <= lb_bytes) *reinterpret_cast<uint4*>(Lb + byte0 + (int64_t)q * 16) = wslab4[q];
        }
    }
    if (mine) ov[word0 + lane] = outo;
    const uint32_t so = es_wave_sum(__popcll(outo));
    if (lane == 0) { co[wave] = so; d0[wave] = delta0; d1[wave] = delta1; }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t z = 0; int32_t x = 0, y = 0;
        for (int q = 0; q < kWordsPerBlock; ++q) { z += co[q]; x += d0[q]; y += d1[q]; }
        bso[blockIdx.x] = z; bd0[blockIdx.x] = x; bd1[blockIdx.x] = y;
    }
}

// One workgroup: ranks of the rejected new nodes, sizes after the admissions (Sp[0..1], Sp[2] = how
// many nodes are to be placed), and the sizes after placing them one by one in the smaller
// partition (0 on a tie): the first |difference| go to the smaller one, the rest alternate 0,1,...
__global__ __launch_bounds__(kBlock) void k_es_scan_spill(int64_t blocks, const uint32_t* bso, uint32_t* boo,
                                                          const int32_t* bd0, const int32_t* bd1, u64* S, long long* Sp)
{
    __shared__ uint32_t wsum[kWordsPerBlock];
    __shared__ long long part0[kWordsPerBlock], part1[kWordsPerBlock];
    const uint32_t total = es_block_scan(bso, boo, blocks, wsum);
    long long x = 0, y = 0;
    for (int64_t i = threadIdx.x; i < blocks; i += kBlock) { x += bd0[i]; y += bd1[i]; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { x += __shfl_down(x, o); y += __shfl_down(y, o); }
    if ((threadIdx.x & 63) == 0) { part0[threadIdx.x >> 6] = x; part1[threadIdx.x >> 6] = y; }
    __syncthreads();
    if (threadIdx.x == 0) {
        long long a = (long long)S[0], b = (long long)S[1];
        for (int q = 0; q < kWordsPerBlock; ++q) { a += part0[q]; b += part1[q]; }
        Sp[0] = a; Sp[1] = b; Sp[2] = (long long)total;
        const long long gap = a <= b ? b - a : a - b;
        const long long lead = (long long)total < gap ? (long long)total : gap;
        const long long rest = (long long)total - lead;
        if (a <= b) a += lead; else b += lead;
        a += (rest + 1) / 2;
        b += rest / 2;
        S[0] = (u64)a; S[1] = (u64)b;
    }
}

__global__ __launch_bounds__(kBlock) void k_es_spill(int64_t words, const u64* __restrict__ ov,
                                                     const uint32_t* __restrict__ boo, const long long* __restrict__ Sp,
                                                     uint8_t* Lb)
{
    if (Sp[2] == 0) return;
    __shared__ uint32_t co[kWordsPerBlock];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t word0 = ((int64_t)blockIdx.x * kWordsPerBlock + wave) * kWaveWords;
    const u64 myo = word0 + lane < words ? ov[word0 + lane] : 0ull;
    const uint32_t p = __popcll(myo);
    const uint32_t ex = es_wave_exclusive(p, lane);
    if (lane == 63) co[wave] = ex + p;
    __syncthreads();
    long long base = boo[blockIdx.x];
    for (int q = 0; q < wave; ++q) base += co[q];
    const long long a = Sp[0], b = Sp[1];
    const long long gap = a <= b ? b - a : a - b;
    for (u64 todo = __ballot(myo != 0ull); todo; todo &= todo - 1ull) {
        const int i = __builtin_ctzll(todo);
        const u64 o = es_bcast(myo, i);
        if ((o >> lane) & 1ull) {
            const long long j = base + __builtin_amdgcn_readlane(ex, i) + __popcll(o & ((1ull << lane) - 1ull));
            const int t = j < gap ? (a <= b ? 0 : 1) : (int)((j - gap) & 1);
            Lb[(word0 + i) * 64 + lane] = (uint8_t)t;
        }
    }
}

__global__ __launch_bounds__(256) void k_es_expand(int64_t n, const uint8_t* __restrict__ Lb, int32_t* parts,
                                                   const u64* S, int64_t* sizes_out)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += stride) {
        const uint32_t l = Lb[v];
        parts[v] = l == kNone ? -1 : (int32_t)l;
    }
    if (sizes_out && blockIdx.x == 0 && threadIdx.x < 2) sizes_out[threadIdx.x] = (int64_t)S[threadIdx.x];
}

// listed edges whose ends carry different labels (Sec. 1)
__global__ __launch_bounds__(256) void k_es_cut(const int32_t* __restrict__ src, const int32_t* __restrict__ dst, int64_t m,
                                                const int32_t* __restrict__ parts, u64* cut)
{
    __shared__ u64 wsum[4];
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    u64 c = 0;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < m; e += stride)
        c += parts[src[e]] != parts[dst[e]];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) c += __shfl_down(c, o);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) {
        const u64 t = wsum[0] + wsum[1] + wsum[2] + wsum[3];
        if (t) atomicAdd(cut, t);
    }
}

// ---- recursive bisection (Sec. 4.1: more than two partitions by splitting every part in two) ------
//
// Per level the edges that still lie inside a group are kept grouped by group, in stream order, and
// already written in the group's own node numbers (0..nv-1 in ascending id), so that a group's
// segment is the input of the two-partition run as it stands.  Per level and group there is also
// the list of its nodes' ids (and their seed bits) in that numbering.  When a group has been split,
// every node gets its number inside its half (its rank among the nodes of the same half), the
// halves' node lists are written, and the group's edges are rewritten in those numbers while they
// are sorted into "both ends in half 0", "both ends in half 1" and "ends part" (dropped).

constexpr int kSelBlock = 1024;     // stable selection of edges: a thread owns kSelPer consecutive edges
constexpr int kSelPer = 4;
constexpr int kSelTile = kSelBlock * kSelPer;

// flag bitmap of a predicate over items 0..count-1 (what = 0: value[i] == key, what = 1: value[i] < 0)
// and the number of flagged items per workgroup of kBlock items
__global__ __launch_bounds__(kBlock) void k_rb_flags(int64_t count, const int32_t* __restrict__ value, int32_t key,
                                                     int what, u64* flag, uint32_t* bsum)
{
    __shared__ uint32_t c[kWordsPerBlock];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    bool on = false;
    if (i < count) { const int32_t x = value[i]; on = what == 0 ? x == key : x < 0; }
    const u64 b = __ballot(on);
    if (lane == 0) {
        const int64_t w = (int64_t)blockIdx.x * kWordsPerBlock + wave;
        if (w * 64 < count) flag[w] = b;
        c[wave] = __popcll(b);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = 0;
        for (int q = 0; q < kWordsPerBlock; ++q) t += c[q];
        bsum[blockIdx.x] = t;
    }
}

// exclusive scan of the per-workgroup counts; the total goes to total_out[0]
__global__ __launch_bounds__(kBlock) void k_rb_scan(int64_t blocks, const uint32_t* bsum, uint32_t* boff, long long* total_out)
{
    __shared__ uint32_t wsum[kWordsPerBlock];
    const uint32_t total = es_block_scan(bsum, boff, blocks, wsum);
    if (threadIdx.x == 0) total_out[0] = (long long)total;
}

// rank of a flagged item among the flagged ones, ascending index
__device__ __forceinline__ uint32_t rb_rank(const u64* __restrict__ flag, const uint32_t* __restrict__ boff,
                                            uint32_t* c /* kWordsPerBlock words of LDS */, int64_t count, bool& on)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t w = (int64_t)blockIdx.x * kWordsPerBlock + wave;
    const u64 word = w * 64 < count ? flag[w] : 0ull;
    if (lane == 0) c[wave] = __popcll(word);
    __syncthreads();
    uint32_t r = boff[blockIdx.x];
    for (int q = 0; q < wave; ++q) r += c[q];
    on = (word >> lane) & 1ull;
    return r + __popcll(word & ((1ull << lane) - 1ull));
}

// Nodes the two-partition run left without a label (no edge inside the group) are placed one by one,
// ascending id, in the currently smaller half (0 on a tie): closed form from the run's sizes, as for
// the spill of the two-partition run.  flag / boff: the unlabelled nodes and their scanned counts.
__global__ __launch_bounds__(kBlock) void k_rb_place(int64_t nv, const u64* __restrict__ flag, const uint32_t* __restrict__ boff,
                                                     int32_t* sub_parts, const int64_t* __restrict__ sub_sizes)
{
    __shared__ uint32_t c[kWordsPerBlock];
    bool on;
    const long long j = rb_rank(flag, boff, c, nv, on);
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= nv || !on) return;
    const long long a = sub_sizes[0], b = sub_sizes[1];
    const long long gap = a <= b ? b - a : a - b;
    sub_parts[i] = j < gap ? (a <= b ? 0 : 1) : (int)((j - gap) & 1);
}

// flag / boff: the nodes of half 0 and their scanned counts; count0[0] = how many.  A node of half b gets
// its number inside the half (its rank among the nodes of the same half); packed[i] = that number with
// the half in bit 31; the halves' node lists (ids and next level's seed bits) are written, half 0 first.
// At the last level the labels 2g + half go out instead.  gof == nullptr: node i has id i.
__global__ __launch_bounds__(kBlock) void k_rb_children(int64_t nv, const u64* __restrict__ flag, const uint32_t* __restrict__ boff,
                                                        const int32_t* __restrict__ sub_parts, const int32_t* __restrict__ gof,
                                                        int32_t g, const long long* __restrict__ count0,
                                                        const int32_t* __restrict__ next_bits, uint32_t* packed,
                                                        int32_t* gof_next, int32_t* seed_next, int32_t* labels_out)
{
    __shared__ uint32_t c[kWordsPerBlock];
    bool on;
    const uint32_t r0 = rb_rank(flag, boff, c, nv, on);      // nodes of half 0 before this one
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= nv) return;
    const int32_t id = gof ? gof[i] : (int32_t)i;
    const uint32_t half = on ? 0u : 1u;
    if (labels_out) { labels_out[id] = 2 * g + (int32_t)half; return; }
    const uint32_t num = on ? r0 : (uint32_t)i - r0;
    packed[i] = num | (half << 31);
    const int64_t at = on ? (int64_t)num : count0[0] + (int64_t)num;
    gof_next[at] = id;
    seed_next[at] = next_bits[id];
}

// An edge of the group goes to the half both its ends are in (key 0 / 1) or is dropped (key 2); its
// ends are rewritten in the halves' node numbers (tmp_s, tmp_d) for the scatter.
__global__ __launch_bounds__(kSelBlock) void k_rb_split_count(int64_t m, const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                                              const uint32_t* __restrict__ packed, uint8_t* __restrict__ key,
                                                              int32_t* __restrict__ tmp_s, int32_t* __restrict__ tmp_d,
                                                              uint32_t* bc0, uint32_t* bc1)
{
    __shared__ uint32_t c0[kSelBlock / 64], c1[kSelBlock / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t e0 = (int64_t)blockIdx.x * kSelTile + (int64_t)threadIdx.x * kSelPer;
    uint32_t n0 = 0, n1 = 0;
#pragma unroll
    for (int u = 0; u < kSelPer; ++u) {
        const int64_t e = e0 + u;
        if (e < m) {
            const uint32_t a = packed[src[e]], b = packed[dst[e]];
            const int k = (a >> 31) == (b >> 31) ? (int)(a >> 31) : 2;
            key[e] = (uint8_t)k;
            tmp_s[e] = (int32_t)(a & 0x7FFFFFFFu);
            tmp_d[e] = (int32_t)(b & 0x7FFFFFFFu);
            n0 += k == 0; n1 += k == 1;
        }
    }
    n0 = es_wave_sum(n0); n1 = es_wave_sum(n1);
    if (lane == 0) { c0[wave] = n0; c1[wave] = n1; }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t x = 0, y = 0;
        for (int q = 0; q < kSelBlock / 64; ++q) { x += c0[q]; y += c1[q]; }
        bc0[blockIdx.x] = x; bc1[blockIdx.x] = y;
    }
}

__global__ __launch_bounds__(kBlock) void k_rb_split_scan(int64_t blocks, const uint32_t* bc0, const uint32_t* bc1,
                                                          uint32_t* bo0, uint32_t* bo1, long long* totals)
{
    __shared__ uint32_t wsum[kWordsPerBlock];
    const uint32_t t0 = es_block_scan(bc0, bo0, blocks, wsum);
    const uint32_t t1 = es_block_scan(bc1, bo1, blocks, wsum);
    if (threadIdx.x == 0) { totals[0] = (long long)t0; totals[1] = (long long)t1; }
}

// stable: the edges of child 0 (key 0, as k_rb_split_count stored it) keep their order and land from
// at0 on, those of child 1 right after them
__global__ __launch_bounds__(kSelBlock) void k_rb_split_scatter(int64_t m, const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                                                const uint8_t* __restrict__ key,
                                                                const uint32_t* __restrict__ bo0, const uint32_t* __restrict__ bo1,
                                                                int32_t* out_src, int32_t* out_dst, int64_t at0,
                                                                const long long* __restrict__ totals)
{
    __shared__ uint32_t c0[kSelBlock / 64], c1[kSelBlock / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t e0 = (int64_t)blockIdx.x * kSelTile + (int64_t)threadIdx.x * kSelPer;
    int32_t s[kSelPer], d[kSelPer];
    int k[kSelPer];
    uint32_t n0 = 0, n1 = 0;
#pragma unroll
    for (int u = 0; u < kSelPer; ++u) {
        const int64_t e = e0 + u;
        k[u] = 2; s[u] = 0; d[u] = 0;
        if (e < m) {
            s[u] = src[e]; d[u] = dst[e];
            k[u] = key[e];
            n0 += k[u] == 0; n1 += k[u] == 1;
        }
    }
    const uint32_t x0 = es_wave_exclusive(n0, lane), x1 = es_wave_exclusive(n1, lane);
    if (lane == 63) { c0[wave] = x0 + n0; c1[wave] = x1 + n1; }
    __syncthreads();
    int64_t p0 = at0 + bo0[blockIdx.x] + x0, p1 = at0 + totals[0] + bo1[blockIdx.x] + x1;
    for (int q = 0; q < wave; ++q) { p0 += c0[q]; p1 += c1[q]; }
#pragma unroll
    for (int u = 0; u < kSelPer; ++u) {
        if (k[u] == 0) { out_src[p0] = s[u]; out_dst[p0] = d[u]; ++p0; }
        else if (k[u] == 1) { out_src[p1] = s[u]; out_dst[p1] = d[u]; ++p1; }
    }
}

// ---- host side ---------------------------------------------------------------------------------

struct EsProfile {
    std::mutex mu;
    bool on = false;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> count_events;
    int64_t edges = 0;      // edges handed to the timed launches
} es_prof;

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

inline int grid_for(int64_t items, int block, int64_t cap)
{
    int64_t g = (items + block - 1) / block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

}  // namespace

extern "C" {

int grem_edge_stream_bipartition(const int32_t* src, const int32_t* dst, int64_t m, int64_t n,
                                 int64_t c_size, int64_t P, const int32_t* seed_parts, int32_t mode,
                                 int32_t* parts_out, int64_t* sizes_out, double* nbr_counts_out,
                                 void* stream_)
{
    if (!src || !dst || !seed_parts || !parts_out || m < 1 || n < 1 || n > INT32_MAX || c_size < 1 ||
        P < 1 || 2 * P < n || (mode != GREM_EDGE_REFINE && mode != GREM_EDGE_FIXED))
        return GREM_ERR_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    const int64_t words = (n + 63) / 64;
    const int64_t seed_blocks = (words + kWordsPerBlock - 1) / kWordsPerBlock;         // a wave per word
    const int64_t blocks = (words + kWordsPerBlock * kWaveWords - 1) / (kWordsPerBlock * kWaveWords);

    // one stream-ordered allocation, carved up
    size_t off = 0;
    auto carve = [&](size_t bytes) { const size_t at = off; off += align256(bytes); return at; };
    const size_t o_small = carve(256);                       // S[2], Sp[3], flags[2]
    const size_t o_lb = carve((size_t)n);
    const size_t o_hc = carve((size_t)n * 8);
    const size_t o_est = nbr_counts_out ? 0 : carve((size_t)n * 16);
    const size_t o_mark = carve((size_t)words * 8), o_mv0 = carve((size_t)words * 8);
    const size_t o_mv1 = carve((size_t)words * 8), o_ov = carve((size_t)words * 8);
    size_t o_b[8];
    for (int i = 0; i < 8; ++i) o_b[i] = carve((size_t)blocks * 4);
    uint8_t* ws = nullptr;
    if (hipMallocAsync((void**)&ws, off, stream) != hipSuccess) { (void)hipGetLastError(); return GREM_ERR_NOMEM; }
    u64* S = (u64*)(ws + o_small);
    long long* Sp = (long long*)(ws + o_small + 16);
    uint32_t* flags = (uint32_t*)(ws + o_small + 64);
    uint8_t* Lb = ws + o_lb;
    u64* hc = (u64*)(ws + o_hc);
    double2* est = nbr_counts_out ? (double2*)nbr_counts_out : (double2*)(ws + o_est);
    u64 *mark = (u64*)(ws + o_mark), *mv0 = (u64*)(ws + o_mv0), *mv1 = (u64*)(ws + o_mv1), *ov = (u64*)(ws + o_ov);
    uint32_t *bs0 = (uint32_t*)(ws + o_b[0]), *bs1 = (uint32_t*)(ws + o_b[1]), *bso = (uint32_t*)(ws + o_b[2]);
    uint32_t *bo0 = (uint32_t*)(ws + o_b[3]), *bo1 = (uint32_t*)(ws + o_b[4]), *boo = (uint32_t*)(ws + o_b[5]);
    int32_t *bd0 = (int32_t*)(ws + o_b[6]), *bd1 = (int32_t*)(ws + o_b[7]);

    int rc = GREM_OK;
    auto fail = [&](int code) { (void)hipGetLastError(); (void)hipFreeAsync(ws, stream); return code; };
    auto fill = [&](void* p, size_t bytes, u64 value) {
        const size_t count = bytes / 8;
        hipLaunchKernelGGL(k_es_fill64, dim3(grid_for((int64_t)count, 256, 16384)), dim3(256), 0, stream, (u64*)p, count, value);
    };
    fill(ws + o_small, 256, 0ull);
    fill(Lb, align256((size_t)n), ~0ull);
    fill(hc, (size_t)n * 8, 0ull);
    fill(est, (size_t)n * 16, 0ull);
    fill(mark, (size_t)words * 8, 0ull);

    const int egrid_all = grid_for(m, 256, 8192);
    hipLaunchKernelGGL(k_es_check, dim3(egrid_all), dim3(256), 0, stream, src, dst, m, (uint32_t)n, flags);
    // the range check must be known before any kernel indexes with the endpoints
    struct { u64 S[2]; long long Sp[3]; long long pad[3]; uint32_t flags[2]; } host;
    static_assert(sizeof(host) >= 72, "layout");
    if (hipMemcpyAsync(&host, ws + o_small, sizeof(host), hipMemcpyDeviceToHost, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess)
        return fail(GREM_ERR_HIP);
    if (host.flags[0]) return fail(GREM_ERR_ARG);

    if (hipFuncSetAttribute((const void*)k_es_apply, hipFuncAttributeMaxDynamicSharedMemorySize, kBlock * 64) != hipSuccess)
        return fail(GREM_ERR_HIP);
    const int64_t nchunks = (m + c_size - 1) / c_size;
    bool profile;
    { std::lock_guard<std::mutex> lock(es_prof.mu); profile = es_prof.on; }
    for (int64_t i = 0; i < nchunks; ++i) {
        const int64_t lo = i * c_size, hi = (lo + c_size < m) ? lo + c_size : m;
        const int egrid = grid_for((hi - lo + kCountUnroll - 1) / kCountUnroll, kCountBlock, 1 << 20);
        if (i == 0) {
            hipLaunchKernelGGL(k_es_mark, dim3(grid_for(hi - lo, kCountBlock, 8192)), dim3(kCountBlock), 0, stream, src, dst, lo, hi, mark);
            hipLaunchKernelGGL(k_es_seed, dim3((int)seed_blocks), dim3(kBlock), 0, stream, words, mark, seed_parts, Lb, S, flags);
            if (hipMemcpyAsync(&host, ws + o_small, sizeof(host), hipMemcpyDeviceToHost, stream) != hipSuccess ||
                hipStreamSynchronize(stream) != hipSuccess)
                return fail(GREM_ERR_HIP);
            if (host.flags[1] || (long long)host.S[0] > P || (long long)host.S[1] > P) return fail(GREM_ERR_SEED);
        }
        hipEvent_t e0 = nullptr, e1 = nullptr;
        if (profile) {
            // timing only: no system-scope fence when the events complete
            if (hipEventCreateWithFlags(&e0, hipEventDisableSystemFence) != hipSuccess ||
                hipEventCreateWithFlags(&e1, hipEventDisableSystemFence) != hipSuccess)
                return fail(GREM_ERR_HIP);
            (void)hipEventRecord(e0, stream);
        }
        hipLaunchKernelGGL(k_es_count, dim3(egrid), dim3(kCountBlock), 0, stream, src, dst, lo, hi, Lb, mark, hc);
        if (profile) {
            (void)hipEventRecord(e1, stream);
            std::lock_guard<std::mutex> lock(es_prof.mu);
            es_prof.count_events.emplace_back(e0, e1);
            es_prof.edges += hi - lo;
        }
        hipLaunchKernelGGL(k_es_score, dim3((int)blocks), dim3(kBlock), 0, stream, n, words, i == 0 ? 1 : 0,
                           mode == GREM_EDGE_FIXED ? 1 : 0, (long long)P, S, mark, hc, Lb, est, mv0, mv1, bs0, bs1);
        if (i == 0) continue;
        hipLaunchKernelGGL(k_es_scan_movers, dim3(1), dim3(kBlock), 0, stream, blocks, bs0, bs1, bo0, bo1);
        hipLaunchKernelGGL(k_es_apply, dim3((int)blocks), dim3(kBlock), (size_t)kBlock * 64, stream, words, (long long)P, S, mv0,
                           mv1, bo0, bo1, Lb, (int64_t)align256((size_t)n), ov, bso, bd0, bd1);
        hipLaunchKernelGGL(k_es_scan_spill, dim3(1), dim3(kBlock), 0, stream, blocks, bso, boo, bd0, bd1, S, Sp);
        hipLaunchKernelGGL(k_es_spill, dim3((int)blocks), dim3(kBlock), 0, stream, words, ov, boo, Sp, Lb);
    }
    hipLaunchKernelGGL(k_es_expand, dim3(grid_for(n, 256, 16384)), dim3(256), 0, stream, n, Lb, parts_out, S, sizes_out);
    if (hipGetLastError() != hipSuccess) rc = GREM_ERR_HIP;
    if (hipFreeAsync(ws, stream) != hipSuccess) rc = GREM_ERR_HIP;
    return rc;
}

int grem_recursive_bisection(const int32_t* src, const int32_t* dst, int64_t m, int64_t n, int32_t levels,
                             int64_t chunks, double balance_slack, const int32_t* seed_bits, int32_t mode,
                             int32_t* labels_out, void* stream_)
{
    if (!src || !dst || !seed_bits || !labels_out || m < 1 || n < 1 || n > INT32_MAX || levels < 1 || levels > 20 ||
        chunks < 1 || !(balance_slack >= 1.0) || (mode != GREM_EDGE_REFINE && mode != GREM_EDGE_FIXED))
        return GREM_ERR_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    const int64_t node_blocks = (n + kBlock - 1) / kBlock;
    const int64_t sel_blocks = (m + kSelTile - 1) / kSelTile;
    size_t off = 0;
    auto carve = [&](size_t bytes) { const size_t at = off; off += align256(bytes); return at; };
    const size_t o_small = carve(256);                 // totals[3], flags
    size_t o_gof[2], o_seed[2];                        // two generations of the groups' node lists
    for (int i = 0; i < 2; ++i) { o_gof[i] = carve((size_t)n * 4); o_seed[i] = carve((size_t)n * 4); }
    const size_t o_packed = carve((size_t)n * 4);
    const size_t o_parts = carve((size_t)n * 4 + 8), o_sizes = carve(16);
    const size_t o_flag = carve((size_t)((n + 63) / 64) * 8);
    const size_t o_bsum = carve((size_t)node_blocks * 4), o_boff = carve((size_t)node_blocks * 4);
    size_t o_sel[4];
    for (int i = 0; i < 4; ++i) o_sel[i] = carve((size_t)sel_blocks * 4);
    const size_t o_tmps = carve((size_t)m * 4), o_tmpd = carve((size_t)m * 4), o_key = carve((size_t)m);
    size_t o_lev[4];                                   // two generations of the grouped edge list
    for (int i = 0; i < 4; ++i) o_lev[i] = carve((size_t)m * 4);
    uint8_t* ws = nullptr;
    if (hipMallocAsync((void**)&ws, off, stream) != hipSuccess) { (void)hipGetLastError(); return GREM_ERR_NOMEM; }
    auto fail = [&](int code) { (void)hipGetLastError(); (void)hipStreamSynchronize(stream); (void)hipFreeAsync(ws, stream); return code; };
    long long* totals = (long long*)(ws + o_small);    // [0..1] edges kept per half, [2] nodes in half 0
    uint32_t* flags = (uint32_t*)(ws + o_small + 64);
    uint32_t* packed = (uint32_t*)(ws + o_packed);
    int32_t* sub_parts = (int32_t*)(ws + o_parts);
    int64_t* sub_sizes = (int64_t*)(ws + o_sizes);
    u64* flag = (u64*)(ws + o_flag);
    uint32_t *bsum = (uint32_t*)(ws + o_bsum), *boff = (uint32_t*)(ws + o_boff);
    uint32_t *bc0 = (uint32_t*)(ws + o_sel[0]), *bc1 = (uint32_t*)(ws + o_sel[1]);
    uint32_t *bo0 = (uint32_t*)(ws + o_sel[2]), *bo1 = (uint32_t*)(ws + o_sel[3]);
    int32_t *tmp_s = (int32_t*)(ws + o_tmps), *tmp_d = (int32_t*)(ws + o_tmpd);
    uint8_t* key = ws + o_key;

    auto fill = [&](void* p, size_t bytes, u64 value) {
        const size_t count = bytes / 8;
        hipLaunchKernelGGL(k_es_fill64, dim3(grid_for((int64_t)count, 256, 16384)), dim3(256), 0, stream, (u64*)p, count, value);
    };
    struct { long long totals[3]; long long pad[5]; uint32_t flags[2]; } host;
    auto read_small = [&]() {
        return hipMemcpyAsync(&host, ws + o_small, sizeof(host), hipMemcpyDeviceToHost, stream) == hipSuccess &&
               hipStreamSynchronize(stream) == hipSuccess;
    };
    fill(ws + o_small, 256, 0ull);
    hipLaunchKernelGGL(k_es_check, dim3(grid_for(m, 256, 8192)), dim3(256), 0, stream, src, dst, m, (uint32_t)n, flags);
    if (!read_small()) return fail(GREM_ERR_HIP);
    if (host.flags[0]) return fail(GREM_ERR_ARG);

    // level 0: one group, everyone, numbered by id; its edges and seed bits are the inputs themselves
    const int32_t *cur_s = src, *cur_d = dst;
    const int32_t *cur_gof = nullptr, *cur_seed = seed_bits;
    std::vector<int64_t> eoff{0, m}, noff{0, n};
    for (int32_t level = 0; level < levels; ++level) {
        const bool last = level + 1 == levels;
        int32_t* out_s = (int32_t*)(ws + o_lev[(level & 1) * 2]);
        int32_t* out_d = (int32_t*)(ws + o_lev[(level & 1) * 2 + 1]);
        int32_t* gof_next = (int32_t*)(ws + o_gof[level & 1]);
        int32_t* seed_next = (int32_t*)(ws + o_seed[level & 1]);
        const int32_t groups = 1 << level;
        std::vector<int64_t> eoff_next((size_t)2 * groups + 1, 0), noff_next((size_t)2 * groups + 1, 0);
        const int32_t* next_bits = last ? seed_bits : seed_bits + (size_t)(level + 1) * (size_t)n;
        for (int32_t g = 0; g < groups; ++g) {
            const int64_t e_lo = eoff[g], mg = eoff[g + 1] - eoff[g];
            const int64_t v_lo = noff[g], nv = noff[g + 1] - noff[g];
            eoff_next[2 * g + 1] = eoff_next[2 * g + 2] = eoff_next[2 * g];
            noff_next[2 * g + 1] = noff_next[2 * g + 2] = noff_next[2 * g];
            if (nv == 0) continue;
            if (mg > 0) {
                const int64_t c_size = (mg + chunks - 1) / chunks;
                const int64_t P = grem_capacity(nv, 2, balance_slack);
                const int rc = grem_edge_stream_bipartition(cur_s + e_lo, cur_d + e_lo, mg, nv, c_size, P, cur_seed + v_lo, mode,
                                                            sub_parts, sub_sizes, nullptr, stream_);
                if (rc != GREM_OK) return fail(rc);
            } else {
                fill(sub_parts, ((size_t)nv * 4 + 7) & ~(size_t)7, ~0ull);
                fill(sub_sizes, 16, 0ull);
            }
            const int64_t vb = (nv + kBlock - 1) / kBlock;
            // unlabelled nodes are placed
            hipLaunchKernelGGL(k_rb_flags, dim3((int)vb), dim3(kBlock), 0, stream, nv, sub_parts, 0, 1, flag, bsum);
            hipLaunchKernelGGL(k_rb_scan, dim3(1), dim3(kBlock), 0, stream, vb, bsum, boff, totals + 2);
            hipLaunchKernelGGL(k_rb_place, dim3((int)vb), dim3(kBlock), 0, stream, nv, flag, boff, sub_parts, sub_sizes);
            // numbers inside the halves, the halves' node lists (or, at the last level, the labels)
            hipLaunchKernelGGL(k_rb_flags, dim3((int)vb), dim3(kBlock), 0, stream, nv, sub_parts, 0, 0, flag, bsum);
            hipLaunchKernelGGL(k_rb_scan, dim3(1), dim3(kBlock), 0, stream, vb, bsum, boff, totals + 2);
            hipLaunchKernelGGL(k_rb_children, dim3((int)vb), dim3(kBlock), 0, stream, nv, flag, boff, sub_parts,
                               cur_gof ? cur_gof + v_lo : (const int32_t*)nullptr, g, totals + 2, next_bits, packed,
                               gof_next + v_lo, seed_next + v_lo, last ? labels_out : (int32_t*)nullptr);
            if (last) continue;
            // the group's edges that stay inside a half, in the halves' numbers, for the next level
            if (mg > 0) {
                const int64_t sb = (mg + kSelTile - 1) / kSelTile;
                hipLaunchKernelGGL(k_rb_split_count, dim3((int)sb), dim3(kSelBlock), 0, stream, mg, cur_s + e_lo, cur_d + e_lo,
                                   packed, key, tmp_s, tmp_d, bc0, bc1);
                hipLaunchKernelGGL(k_rb_split_scan, dim3(1), dim3(kBlock), 0, stream, sb, bc0, bc1, bo0, bo1, totals);
                hipLaunchKernelGGL(k_rb_split_scatter, dim3((int)sb), dim3(kSelBlock), 0, stream, mg, tmp_s, tmp_d,
                                   key, bo0, bo1, out_s, out_d, eoff_next[2 * g], totals);
            } else {
                fill(totals, 16, 0ull);
            }
            if (!read_small()) return fail(GREM_ERR_HIP);
            eoff_next[2 * g + 1] = eoff_next[2 * g] + host.totals[0];
            eoff_next[2 * g + 2] = eoff_next[2 * g + 1] + host.totals[1];
            noff_next[2 * g + 1] = noff_next[2 * g] + host.totals[2];
            noff_next[2 * g + 2] = noff_next[2 * g] + nv;
        }
        cur_s = out_s; cur_d = out_d;
        cur_gof = gof_next; cur_seed = seed_next;
        eoff.swap(eoff_next);
        noff.swap(noff_next);
    }
    int rc = hipGetLastError() == hipSuccess ? GREM_OK : GREM_ERR_HIP;
    if (hipFreeAsync(ws, stream) != hipSuccess) rc = GREM_ERR_HIP;
    return rc;
}

int grem_edge_list_cut(const int32_t* src, const int32_t* dst, int64_t m, const int32_t* parts,
                       int64_t* cut_out, void* stream_)
{
    if (!src || !dst || !parts || !cut_out || m < 0) return GREM_ERR_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    hipLaunchKernelGGL(k_es_fill64, dim3(1), dim3(256), 0, stream, (u64*)cut_out, (size_t)1, 0ull);
    if (m > 0)
        hipLaunchKernelGGL(k_es_cut, dim3(grid_for(m, 256, 8192)), dim3(256), 0, stream, src, dst, m, parts, (u64*)cut_out);
    return hipGetLastError() == hipSuccess ? GREM_OK : GREM_ERR_HIP;
}

int grem_edge_stream_profile_enable(int32_t on)
{
    std::lock_guard<std::mutex> lock(es_prof.mu);
    es_prof.on = on != 0;
    return GREM_OK;
}

int grem_edge_stream_profile_read(double* count_ms, int64_t* launches, int64_t* edges)
{
    std::lock_guard<std::mutex> lock(es_prof.mu);
    double total = 0.0;
    int rc = GREM_OK;
    for (auto& ev : es_prof.count_events) {
        float ms = 0.f;
        if (hipEventSynchronize(ev.second) != hipSuccess || hipEventElapsedTime(&ms, ev.first, ev.second) != hipSuccess)
            rc = GREM_ERR_HIP;
        total += ms;
        (void)hipEventDestroy(ev.first);
        (void)hipEventDestroy(ev.second);
    }
    if (count_ms) *count_ms = total;
    if (launches) *launches = (int64_t)es_prof.count_events.size();
    if (edges) *edges = es_prof.edges;
    es_prof.count_events.clear();
    es_prof.edges = 0;
    return rc;
}

}  // extern "C"
