// Expected number of edge cuts of fixed greedy decisions made from a fraction x of the edges, for gfx950
// (Armada paper, Sec. 4.2, Eq. (1)): for a two-way labelling, node i has k_i labelled neighbours, k0_i of
// them in the partition that holds more; with d_i = floor(k_i x + 0.5) of its edges in hand the greedy
// decision is wrong with probability q_i = Pr(K < d_i / 2), K ~ Hypergeometric(k_i, k0_i, d_i), and
//   E[C] = sum_i (k_i - k0_i) (1 - q_i) + k0_i q_i.
// Refinement over two chunks is the same expression at 2x (Sec. 4.2, "The Benefit of Refinement").
//
// Sixteen lanes per node count its CSR row's labels; one of them then sums the tail of the distribution
// term by term: in the log domain (first term from lgamma, the following ones by the ratio of consecutive
// probabilities), or, for a node with few draws, as plain products of ratios.  Sums are reduced per
// workgroup and then by one workgroup in a fixed order, so the result is reproducible.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>

#include "grem.h"

// Per-workgroup partial sums of the entry point that allocates nothing (grem_expected_cut_noalloc).
// One copy per GPU, held until the process ends; host code reaches it only through the address
// hipGetSymbolAddress returns for the current device, never through this name.
constexpr int64_t kXcStaticBlocks = 262144;        // 4 MiB: two doubles per workgroup
static __device__ __align__(256) double scratch[2 * kXcStaticBlocks];

namespace {

constexpr int kXcBlock = 256;

__device__ __forceinline__ double xc_log_choose(double a, double b)
{
    return lgamma(a + 1.0) - lgamma(b + 1.0) - lgamma(a - b + 1.0);
}

constexpr long long kXcFewDraws = 256;     // up to this many draws the tail is summed without logarithms

// One node's terms of Eq. (1) from its two neighbour counts: *ec = (k - k0)(1 - q) + k0 q, *base = k - k0
// (both left as they are for a node without labelled neighbours).
__device__ __forceinline__ void xc_node_terms(uint32_t c0, uint32_t c1, double x, double* ec_out, double* base_out)
{
    const long long k = (long long)c0 + c1, k0 = c0 > c1 ? c0 : c1, r = k - k0;
    if (k <= 0) return;
    long long d = (long long)floor((double)k * x + 0.5);
    if (d > k) d = k;
    if (d < 0) d = 0;
    // q = sum of pmf(j) over the support with 2j < d
    const long long jlo = d - r > 0 ? d - r : 0;
    long long jhi = (d + 1) / 2 - 1;
    if (jhi > k0) jhi = k0;
    double q = 0.0;
    if (jhi >= jlo && jlo == 0 && d <= kXcFewDraws) {
        // few draws, all of which the minority could fill (the usual node at small x): pmf(0) = C(r, d) / C(k, d)
        // as a product of d ratios, the following terms by the ratio of consecutive probabilities -- no
        // lgamma, log or exp.  pmf(0) is about (r/k)^d: whenever the tail is not negligible (at least
        // 1e-20, which takes (r/k)^(d/2) 2^d >= 1e-20) it stays above 1e-40 / 4^d, far from the smallest
        // double for d <= 256; where pmf(0) does underflow, the tail is zero to every digit that counts.
        // (the factors are small integers held in doubles and stepped by one: exact, and no 64-bit
        // integer-to-double conversions in the loops)
        double p = 1.0, rr = (double)r, kk = (double)k;
        for (int i = 0; i < (int)d; ++i) { p *= rr / kk; rr -= 1.0; kk -= 1.0; }
        q = p;
        double a = (double)k0, b = (double)d, c = 1.0, e = (double)(r - d + 1);
        for (int j = 0; j < (int)jhi; ++j) {
            p *= (a * b) / (c * e);
            q += p;
            a -= 1.0; b -= 1.0; c += 1.0; e += 1.0;
        }
        if (q > 1.0) q = 1.0;
    } else if (jhi >= jlo) {
        double logp = xc_log_choose((double)k0, (double)jlo) + xc_log_choose((double)r, (double)(d - jlo)) -
                      xc_log_choose((double)k, (double)d);
        q = exp(logp);
        for (long long j = jlo; j < jhi; ++j) {
            // pmf(j+1) / pmf(j)
            logp += log((double)(k0 - j)) + log((double)(d - j)) - log((double)(j + 1)) - log((double)(r - d + j + 1));
            q += exp(logp);
        }
        if (q > 1.0) q = 1.0;
    }
    *ec_out = (double)r * (1.0 - q) + (double)k0 * q;
    *base_out = (double)r;
}

constexpr int kXcGroup = 16;                       // lanes that share one node's row
constexpr int kXcRows = kXcBlock / kXcGroup;       // nodes per workgroup

template <typename RowT>
__global__ __launch_bounds__(kXcBlock) void k_xc_terms(const RowT* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                                                       int64_t n, const int32_t* __restrict__ labels, double x,
                                                       double* partial_ec, double* partial_base)
{
    __shared__ double s_ec[kXcBlock / 64], s_base[kXcBlock / 64];
    const int sub = threadIdx.x & (kXcGroup - 1);
    const int64_t v = (int64_t)blockIdx.x * kXcRows + threadIdx.x / kXcGroup;
    double ec = 0.0, base = 0.0;
    uint32_t c0 = 0, c1 = 0;
    if (v < n) {
        // (four entries per lane and turn, their loads side by side: a label look-up is a cache miss)
        const int64_t end = (int64_t)rowptr[v + 1];
        constexpr int kTurn = 4;
        for (int64_t e = (int64_t)rowptr[v] + sub; e < end; e += kTurn * kXcGroup) {
            int32_t c[kTurn], l[kTurn];
#pragma unroll
            for (int u = 0; u < kTurn; ++u) c[u] = e + u * kXcGroup < end ? colidx[e + u * kXcGroup] : -1;
#pragma unroll
            for (int u = 0; u < kTurn; ++u) l[u] = c[u] >= 0 ? labels[c[u]] : -1;
#pragma unroll
            for (int u = 0; u < kTurn; ++u) { c0 += l[u] == 0; c1 += l[u] == 1; }
        }
    }
#pragma unroll
    for (int o = kXcGroup / 2; o > 0; o >>= 1) { c0 += __shfl_xor(c0, o); c1 += __shfl_xor(c1, o); }
    if (v < n && sub == 0) xc_node_terms(c0, c1, x, &ec, &base);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { ec += __shfl_down(ec, o); base += __shfl_down(base, o); }
    if ((threadIdx.x & 63) == 0) { s_ec[threadIdx.x >> 6] = ec; s_base[threadIdx.x >> 6] = base; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double a = 0.0, b = 0.0;
        for (int q = 0; q < kXcBlock / 64; ++q) { a += s_ec[q]; b += s_base[q]; }
        partial_ec[blockIdx.x] = a; partial_base[blockIdx.x] = b;
    }
}

// The same terms from neighbour counts that are at hand (counts[2 v], counts[2 v + 1]: the labelled
// neighbours of node v in partition 0 and 1), one lane per node.
constexpr int kXcCountRows = kXcBlock;
__global__ __launch_bounds__(kXcBlock) void k_xc_terms_counts(const uint32_t* __restrict__ counts, int64_t n, double x,
                                                              double* partial_ec, double* partial_base)
{
    __shared__ double s_ec[kXcBlock / 64], s_base[kXcBlock / 64];
    const int64_t v = (int64_t)blockIdx.x * kXcCountRows + threadIdx.x;
    double ec = 0.0, base = 0.0;
    if (v < n) {
        const uint2 c = *reinterpret_cast<const uint2*>(counts + 2 * v);
        xc_node_terms(c.x, c.y, x, &ec, &base);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { ec += __shfl_down(ec, o); base += __shfl_down(base, o); }
    if ((threadIdx.x & 63) == 0) { s_ec[threadIdx.x >> 6] = ec; s_base[threadIdx.x >> 6] = base; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double a = 0.0, b = 0.0;
        for (int q = 0; q < kXcBlock / 64; ++q) { a += s_ec[q]; b += s_base[q]; }
        partial_ec[blockIdx.x] = a; partial_base[blockIdx.x] = b;
    }
}

__global__ __launch_bounds__(1024) void k_xc_total(const double* __restrict__ partial_ec, const double* __restrict__ partial_base,
                                                   int64_t blocks, double* out)
{
    __shared__ double s_ec[16], s_base[16];
    double a = 0.0, b = 0.0;
    for (int64_t i = threadIdx.x; i < blocks; i += 1024) { a += partial_ec[i]; b += partial_base[i]; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { a += __shfl_down(a, o); b += __shfl_down(b, o); }
    if ((threadIdx.x & 63) == 0) { s_ec[threadIdx.x >> 6] = a; s_base[threadIdx.x >> 6] = b; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double x = 0.0, y = 0.0;
        for (int q = 0; q < 16; ++q) { x += s_ec[q]; y += s_base[q]; }
        out[0] = x; out[1] = y;
    }
}

template <typename RowT>
void xc_launch(const void* rowptr, const int32_t* colidx, int64_t n, const int32_t* labels, double x, double* partial,
               int64_t blocks, double* out, hipStream_t stream)
{
    hipLaunchKernelGGL(k_xc_terms<RowT>, dim3((unsigned)blocks), dim3(kXcBlock), 0, stream, (const RowT*)rowptr, colidx, n,
                       labels, x, partial, partial + blocks);
    hipLaunchKernelGGL(k_xc_total, dim3(1), dim3(1024), 0, stream, partial, partial + blocks, blocks, out);
}

constexpr int kXcMaxDevices = 64;
std::mutex xc_mu;
double* xc_scratch_ptr[kXcMaxDevices] = {};        // device address of `scratch`, per GPU

}  // namespace

extern "C" int64_t grem_expected_cut_noalloc_max_n(void) { return kXcStaticBlocks * kXcRows; }

extern "C" int grem_expected_cut_noalloc(const void* rowptr, int32_t rowptr_bits, const int32_t* colidx, int64_t n,
                                         const int32_t* labels, double x, double* out, void* stream_)
{
    if (!rowptr || !colidx || !labels || !out || n < 1 || (rowptr_bits != 32 && rowptr_bits != 64) || !(x > 0.0) ||
        !(x <= 1.0))
        return GREM_ERR_ARG;
    if (n > kXcStaticBlocks * kXcRows) return GREM_ERR_LIMIT;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return GREM_ERR_HIP;
    if (dev < 0 || dev >= kXcMaxDevices) return GREM_ERR_LIMIT;
    double* partial = nullptr;
    {
        std::lock_guard<std::mutex> lock(xc_mu);
        if (!xc_scratch_ptr[dev]) {          // first call on this GPU: look its copy of the array up
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
                (void)hipGetLastError();
                return GREM_ERR_HIP;
            }
            xc_scratch_ptr[dev] = (double*)p;
        }
        partial = xc_scratch_ptr[dev];
    }
    // every workgroup writes its own two slots and the reduction reads exactly those: nothing has to
    // start at zero, whatever an earlier call left behind
    hipStream_t stream = (hipStream_t)stream_;
    const int64_t blocks = (n + kXcRows - 1) / kXcRows;
    if (rowptr_bits == 64) xc_launch<int64_t>(rowptr, colidx, n, labels, x, partial, blocks, out, stream);
    else xc_launch<int32_t>(rowptr, colidx, n, labels, x, partial, blocks, out, stream);
    return hipGetLastError() == hipSuccess ? GREM_OK : GREM_ERR_HIP;
}

extern "C" int grem_expected_cut(const void* rowptr, int32_t rowptr_bits, const int32_t* colidx, int64_t n,
                                 const int32_t* labels, double x, double* out, void* stream_)
{
    if (!rowptr || !colidx || !labels || !out || n < 1 || n > INT32_MAX || (rowptr_bits != 32 && rowptr_bits != 64) ||
        !(x > 0.0) || !(x <= 1.0))
        return GREM_ERR_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    const int64_t blocks = (n + kXcRows - 1) / kXcRows;
    double* partial = nullptr;
    if (hipMallocAsync((void**)&partial, (size_t)blocks * 2 * sizeof(double), stream) != hipSuccess) {
        (void)hipGetLastError();
        return GREM_ERR_NOMEM;
    }
    if (rowptr_bits == 64) xc_launch<int64_t>(rowptr, colidx, n, labels, x, partial, blocks, out, stream);
    else xc_launch<int32_t>(rowptr, colidx, n, labels, x, partial, blocks, out, stream);
    int rc = hipGetLastError() == hipSuccess ? GREM_OK : GREM_ERR_HIP;
    if (hipFreeAsync(partial, stream) != hipSuccess) rc = GREM_ERR_HIP;
    return rc;
}

// Eq. (1) on a plan: the neighbour counts come from the plan's re-laid-out copy of the entries (every label
// look-up served from LDS) instead of one look-up through the caches per CSR entry.
extern "C" int grem_plan_expected_cut(const grem_plan* plan, const int32_t* labels, double x, double* out, void* stream_)
{
    const int64_t n = grem_plan_n(plan);
    if (!plan || n < 1 || !labels || !out || !(x > 0.0) || !(x <= 1.0)) return GREM_ERR_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    const int64_t blocks = (n + kXcCountRows - 1) / kXcCountRows;
    uint32_t* counts = nullptr;
    double* partial = nullptr;
    if (hipMallocAsync((void**)&counts, (size_t)n * 2 * sizeof(uint32_t), stream) != hipSuccess) {
        (void)hipGetLastError();
        return GREM_ERR_NOMEM;
    }
    if (hipMallocAsync((void**)&partial, (size_t)blocks * 2 * sizeof(double), stream) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFreeAsync(counts, stream);
        return GREM_ERR_NOMEM;
    }
    int rc = grem_plan_neighbour_counts(plan, 2, labels, counts, stream);
    if (rc == GREM_OK) {
        hipLaunchKernelGGL(k_xc_terms_counts, dim3((unsigned)blocks), dim3(kXcBlock), 0, stream, (const uint32_t*)counts, n, x,
                           partial, partial + blocks);
        hipLaunchKernelGGL(k_xc_total, dim3(1), dim3(1024), 0, stream, partial, partial + blocks, blocks, out);
        if (hipGetLastError() != hipSuccess) rc = GREM_ERR_HIP;
    }
    if (hipFreeAsync(partial, stream) != hipSuccess) rc = rc == GREM_OK ? GREM_ERR_HIP : rc;
    if (hipFreeAsync(counts, stream) != hipSuccess) rc = rc == GREM_OK ? GREM_ERR_HIP : rc;
    return rc;
}
