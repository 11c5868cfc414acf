// Storing messages as cliques (Section II-A) and the per-cluster summary rows of W.
#include "gbnn_internal.h"

namespace gbnn {
namespace {

// One thread per (message m, cluster c): validates the message, then sets, in the row of the
// active neuron of cluster c, the bits of the message's active neurons of all other clusters.
// Bit sets are idempotent atomic ORs, so the result is independent of thread order.
__global__ __launch_bounds__(256) void k_store(uint32_t *W, int C, int L, int nw,
                                               const int32_t *__restrict__ msgs, int64_t M,
                                               int32_t *__restrict__ status)
{
    const int64_t total = M * C;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += stride) {
        const int64_t m = t / C;
        const int c = (int)(t - m * C);
        const int32_t *sym = msgs + m * C;
        bool ok = true;
        for (int c2 = 0; c2 < C; ++c2) {
            const int32_t s = sym[c2];
            ok = ok && (s >= 0) && (s < L);
        }
        if (!ok) {
            if (c == 0 && status) atomicOr(status, 1);
            continue;
        }
        uint32_t *row = W + ((int64_t)c * L + sym[c]) * nw;
        for (int c2 = 0; c2 < C; ++c2) {
            if (c2 == c) continue;
            const int col = c2 * L + sym[c2];
            const uint32_t bit = 1u << (col & 31);
            uint32_t *p = row + (col >> 5);
            // A stale read can only cause a redundant OR, never a missed one.
            if (!(*p & bit)) atomicOr(p, bit);
        }
    }
}

// Bits of word w (neurons 32w .. 32w+31) that lie in cluster c = neurons [c*L, (c+1)*L).
__device__ __forceinline__ uint32_t own_mask(int c, int L, int w)
{
    int lo = c * L - 32 * w, hi = lo + L;
    if (lo < 0) lo = 0;
    if (hi > 32) hi = 32;
    if (hi <= lo) return 0u;
    const uint32_t upto_hi = (hi == 32) ? 0xFFFFFFFFu : ((1u << hi) - 1u);
    return upto_hi & ~((1u << lo) - 1u);
}

// Cluster summary: has[c][w] = own bits of c | OR over the L rows j of cluster c of W[j][w], i.e.
// bit i says that neuron i is in c or has at least one neighbour in c.  It is what a fully active
// cluster (the sum-of-max initialisation of an erased cluster, Section III-C) lets survive.
// Block = (cluster c, 64 consecutive words), 1024 threads = 16 row subsets x 64 words.
constexpr int kSumRows = 16;
__global__ __launch_bounds__(64 * kSumRows) void k_cluster_summary(const uint32_t *__restrict__ W, int C, int L,
                                                                   int nw, uint32_t *__restrict__ has)
{
    __shared__ uint32_t part[kSumRows][64];
    const int c = blockIdx.y;
    const int wl = threadIdx.x & 63;
    const int r = threadIdx.x >> 6;
    const int w = blockIdx.x * 64 + wl;
    uint32_t acc = 0;
    if (w < nw) {
        const uint32_t *base = W + (int64_t)c * L * nw + w;
        for (int l = r; l < L; l += kSumRows) acc |= base[(int64_t)l * nw];
    }
    part[r][wl] = acc;
    __syncthreads();
    if (r == 0 && w < nw) {
        for (int k = 1; k < kSumRows; ++k) acc |= part[k][wl];
        has[(int64_t)c * nw + w] = acc | own_mask(c, L, w);
    }
}

// full = bit c set iff the summary row of cluster c has every neuron's bit: then every neuron has a
// neighbour in c (or is in c), and a fully active cluster c switches nobody off.  One wave; lane c checks
// row c.  With the densities the method works at this is the rule, and retrieval skips those rows.
__global__ __launch_bounds__(64) void k_summary_full(const uint32_t *__restrict__ has, int C, int n, int nw,
                                                     uint64_t *__restrict__ full)
{
    const int c = threadIdx.x;
    bool all = c < C;
    if (c < C) {
        const uint32_t *row = has + (int64_t)c * nw;
        for (int w = 0; w < nw; ++w) {
            const int bits = n - 32 * w;  // neurons in this word
            const uint32_t need = bits >= 32 ? 0xFFFFFFFFu : ((1u << bits) - 1u);
            all = all && (row[w] & need) == need;
        }
    }
    const uint64_t m = __ballot(all);
    if (c == 0) *full = m;
}

// Wb = W with the intra-cluster blocks set to all ones: row j gets the bits of j's own cluster.
// Also fills the all-zero row `zero_row` of the table and the all-one row that follows it.
__global__ __launch_bounds__(256) void k_fill_blocks(const uint32_t *__restrict__ W, int L, int nw, int64_t words,
                                                     uint32_t *__restrict__ Wb, uint32_t *__restrict__ zero_row)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < nw; t += stride) {
        zero_row[t] = 0u;
        zero_row[nw + t] = 0xFFFFFFFFu;
    }
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < words; t += stride) {
        const int j = (int)(t / nw);
        const int w = (int)(t - (int64_t)j * nw);
        Wb[t] = W[t] | own_mask(j / L, L, w);
    }
}

}  // namespace

hipError_t launch_store(uint32_t *W, int C, int L, int nw, const int32_t *msgs, int64_t M, int32_t *status,
                        hipStream_t s)
{
    if (M == 0) return hipSuccess;
    const int64_t total = M * C;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(k_store, dim3((unsigned)blocks), dim3(256), 0, s, W, C, L, nw, msgs, M, status);
    return hipGetLastError();
}

hipError_t launch_prepare(const uint32_t *W, int C, int L, int nw, uint32_t *has, uint32_t *Wb, uint64_t *full,
                          hipStream_t s)
{
    dim3 grid((unsigned)((nw + 63) / 64), (unsigned)C);
    hipLaunchKernelGGL(k_cluster_summary, grid, dim3(64 * kSumRows), 0, s, W, C, L, nw, has);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_summary_full, dim3(1), dim3(64), 0, s, has, C, C * L, nw, full);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t words = (int64_t)C * L * nw;
    int64_t blocks = (words + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(k_fill_blocks, dim3((unsigned)blocks), dim3(256), 0, s, W, L, nw, words, Wb,
                       Wb + ((int64_t)C * L + C) * nw);
    return hipGetLastError();
}

}  // namespace gbnn
