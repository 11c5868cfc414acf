// Storing messages as cliques (Section II-A) and the per-cluster summary rows of W.
#include "gbnn_device.h"
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

// Storing into W and into an already prepared table at once (a few messages between retrievals): the
// thread of (message m, cluster c) sets, for the message's neuron a of cluster c and its neuron b of every
// other cluster, bit b of row a in W and in the table's copy of W, and bit b of the summary row of cluster
// c (b now has a neighbour in c).  The own-cluster blocks and own bits of the table stay as they are.
// The table is in the layout of the padded network (clusters of Lp neurons, rows of nwp words); hasc, if
// not null, is the copy of the summaries in the canonical layout.
__global__ __launch_bounds__(256) void k_store_update(uint32_t *W, uint32_t *Wb, uint32_t *has, uint32_t *hasc, int C, int L,
                                                      int nw, int Lp, int nwp, const int32_t *__restrict__ msgs, int64_t M,
                                                      int32_t *__restrict__ status)
{
    const int64_t total = M * C;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += stride) {
        const int64_t m = t / C;
        const int c = (int)(t - m * C);
        const int32_t *sym = msgs + m * C;
        bool ok = true;
        for (int c2 = 0; c2 < C; ++c2) ok = ok && (uint32_t)sym[c2] < (uint32_t)L;
        if (!ok) {
            if (c == 0 && status) atomicOr(status, 1);
            continue;
        }
        const int64_t row = ((int64_t)c * L + sym[c]) * nw;
        const int64_t rowp = ((int64_t)c * Lp + sym[c]) * nwp;
        for (int c2 = 0; c2 < C; ++c2) {
            if (c2 == c) continue;
            const int col = c2 * L + sym[c2], colp = c2 * Lp + sym[c2];
            const uint32_t bit = 1u << (col & 31), bitp = 1u << (colp & 31);
            const int w = col >> 5, wp = colp >> 5;
            if (!(W[row + w] & bit)) atomicOr(W + row + w, bit);
            if (!(Wb[rowp + wp] & bitp)) atomicOr(Wb + rowp + wp, bitp);
            if (!(has[(int64_t)c * nwp + wp] & bitp)) atomicOr(has + (int64_t)c * nwp + wp, bitp);
            if (hasc && !(hasc[(int64_t)c * nw + w] & bit)) atomicOr(hasc + (int64_t)c * nw + w, bit);
        }
    }
}

// The same result for many messages, without global atomics.  A workgroup owns the rows of R
// consecutive neurons of one cluster c and builds them in LDS, then ORs the non-zero words into W with
// plain loads and stores -- no other workgroup of the launch touches those rows.  Every wave scans its
// share of the symbol column of cluster c and queues the messages whose symbol falls among the
// workgroup's neurons; whenever 64 or more are queued, the wave walks the queued messages with one lane
// per (message, cluster) pair -- consecutive lanes read consecutive symbols -- and sets the pair's bit
// with an LDS atomic.  A message with a symbol outside [0,L) is skipped by every workgroup that meets it
// and reported by the first workgroup of the cluster the bad symbol is in.
constexpr int kStoreThreads = 1024;
constexpr int kStoreWaves = kStoreThreads / 64;
constexpr int kStoreUnroll = 8;   // symbol loads in flight per lane: the scan is a chain of round trips otherwise
constexpr int kStoreQueue = 128;  // per wave: fewer than 64 left over plus at most 64 new ones
constexpr int kStoreLdsBytes = 64 * 1024 - kStoreWaves * kStoreQueue * 4;  // what is left for the rows

// kPow2: C is a power of two (it then divides 64, and a message's C pairs sit in one wave instruction, so
// its validity is one ballot); otherwise the lane that queues a message checks all of its symbols first.
template <bool kPow2>
__global__ __launch_bounds__(kStoreThreads) void k_store_rows(uint32_t *W, int C, int L, int nw, int R,
                                                              int blocks_per_cluster,
                                                              const int32_t *__restrict__ msgs, int64_t M,
                                                              int32_t *__restrict__ status)
{
    extern __shared__ uint32_t lds[];
    uint32_t *rows = lds;  // [R][nw]
    const int lane = threadIdx.x & 63;
    uint32_t *queue = lds + R * nw + (threadIdx.x >> 6) * kStoreQueue;
    const int c = blockIdx.x / blocks_per_cluster;
    const int b = blockIdx.x - c * blocks_per_cluster;
    const int l0 = b * R;
    const int l1 = l0 + R < L ? l0 + R : L;
    const int words = (l1 - l0) * nw;
    const int lgC = __builtin_ctz((unsigned)C);  // used when kPow2
    for (int t = threadIdx.x; t < words; t += kStoreThreads) rows[t] = 0u;
    __syncthreads();

    int cnt = 0;  // queued messages of this wave (the same in every lane)
    auto flush = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int pairs = cnt * C;
        for (int p0 = 0; p0 < pairs; p0 += 64) {
            const int p = p0 + lane;
            const bool in = p < pairs;
            const int q = !in ? 0 : kPow2 ? p >> lgC : p / C;
            const int c2 = p - q * C;
            const int32_t *sym = msgs + (int64_t)queue[q] * C;
            const int32_t s2 = in ? sym[c2] : 0;
            const int32_t sc = sym[c];  // within [l0, l1): checked when queued
            bool ok = in;
            if (kPow2) {
                const uint64_t bad_lanes = ballot(in && (uint32_t)s2 >= (uint32_t)L);
                const uint64_t mine = C == 64 ? ~0ull : ((1ull << C) - 1ull) << (lane - c2);
                ok = ok && (bad_lanes & mine) == 0;
            }
            if (ok && c2 != c) {
                const int col = c2 * L + s2;
                atomicOr(rows + (sc - l0) * nw + (col >> 5), 1u << (col & 31));
            }
        }
        cnt = 0;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };

    bool bad = false;
    for (int64_t base = 0; base < M; base += (int64_t)kStoreThreads * kStoreUnroll) {
        int32_t s[kStoreUnroll];
#pragma unroll
        for (int u = 0; u < kStoreUnroll; ++u) {
            const int64_t m = base + u * kStoreThreads + threadIdx.x;
            s[u] = m < M ? msgs[m * C + c] : l1;  // l1: outside this block, yet not a bad symbol
        }
#pragma unroll
        for (int u = 0; u < kStoreUnroll; ++u) {
            const int64_t m = base + u * kStoreThreads + threadIdx.x;
            if (m < M && (uint32_t)s[u] >= (uint32_t)L) bad = bad || b == 0;
            bool match = m < M && s[u] >= l0 && s[u] < l1;
            if (!kPow2 && match) {
                const int32_t *sym = msgs + m * C;
                for (int c2 = 0; c2 < C; ++c2) match = match && (uint32_t)sym[c2] < (uint32_t)L;
            }
            const uint64_t takers = ballot(match);
            if (takers) {
                if (match) queue[cnt + (int)mbcnt(takers)] = (uint32_t)m;
                cnt += __builtin_popcountll(takers);
                if (cnt >= 64) flush();
            }
        }
    }
    if (cnt) flush();
    if (bad && status) atomicOr(status, 1);
    __syncthreads();
    uint32_t *out = W + ((int64_t)c * L + l0) * nw;
    for (int t = threadIdx.x; t < words; t += kStoreThreads) {
        const uint32_t v = rows[t];
        if (v) {
            const uint32_t old = out[t];
            if (v & ~old) out[t] = old | v;
        }
    }
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
// neighbour in c (or is in c), and a fully active cluster c switches nobody off.  With the densities the
// method works at this is the rule, and retrieval skips those rows.  One workgroup of 16 waves; a wave
// checks the rows of clusters wave, wave + 16, ..., its lanes striding over the words.  The rows may be in
// the layout of a padded network (clusters of Lp >= L neurons, Lp a multiple of 32): only the first L
// neurons of a cluster exist.  The other 31 words of the 256-byte block of flags are set to zero.
__global__ __launch_bounds__(1024) void k_summary_full(const uint32_t *__restrict__ has, int C, int L, int Lp, int n, int nw,
                                                       uint64_t *__restrict__ full)
{
    __shared__ uint32_t row_full[GBNN_MAX_C];
    const int lane = threadIdx.x & 63;
    for (int c = threadIdx.x >> 6; c < C; c += 16) {
        const uint32_t *row = has + (int64_t)c * nw;
        bool all = true;
        for (int w = lane; w < nw; w += 64) {
            int bits = n - 32 * w;  // neurons in this word
            if (Lp != L) bits = L - 32 * (w % (Lp / 32));
            const uint32_t need = bits >= 32 ? 0xFFFFFFFFu : bits <= 0 ? 0u : ((1u << bits) - 1u);
            all = all && (row[w] & need) == need;
        }
        const bool every = ballot(!all) == 0;
        if (lane == 0) row_full[c] = every ? 1u : 0u;
    }
    __syncthreads();
    if (threadIdx.x < 64) {
        const uint64_t m = ballot(lane < C && row_full[lane < C ? lane : 0] != 0u);
        if (lane == 0) *full = m;
        if (lane >= 1 && lane < 32) full[lane] = 0ull;
    }
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

// The table of a padded network from the canonical W: row c*Lp + l (l < L) gets, for every padded cluster
// c2, the L bits of row c*L + l of W that belong to c2 (all ones for c2 = c), 32 at a time from two
// neighbouring words of W; rows and bits of neurons that do not exist are zero.  Also fills the all-zero
// row of the table and the all-one row that follows it.
__global__ __launch_bounds__(256) void k_fill_padded(const uint32_t *__restrict__ W, int L, int nw, int Lp, int nwp,
                                                     int64_t words, uint32_t *__restrict__ Wb,
                                                     uint32_t *__restrict__ zero_row)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int wpc = Lp / 32;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < nwp; t += stride) {
        zero_row[t] = 0u;
        zero_row[nwp + t] = 0xFFFFFFFFu;
    }
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < words; t += stride) {
        const int jp = (int)(t / nwp);
        const int wp = (int)(t - (int64_t)jp * nwp);
        const int c = jp / Lp, l = jp - c * Lp;
        const int c2 = wp / wpc, l2 = (wp - c2 * wpc) * 32;  // this word: neurons l2 .. l2 + 31 of cluster c2
        uint32_t out = 0u;
        if (l < L && l2 < L) {
            const int count = L - l2 < 32 ? L - l2 : 32;
            const uint32_t keep = count == 32 ? 0xFFFFFFFFu : ((1u << count) - 1u);
            if (c2 == c) {
                out = keep;
            } else {
                const int bit = c2 * L + l2;  // first of `count` consecutive bits of the canonical row
                const uint32_t *row = W + (int64_t)(c * L + l) * nw;
                const int w0 = bit >> 5, sh = bit & 31;
                uint32_t lo = row[w0] >> sh;
                if (sh && w0 + 1 < nw) lo |= row[w0 + 1] << (32 - sh);
                out = lo & keep;
            }
        }
        Wb[t] = out;
    }
}

}  // namespace

hipError_t launch_store(uint32_t *W, int C, int L, int nw, const int32_t *msgs, int64_t M, int32_t *status,
                        int path, hipStream_t s)
{
    if (M == 0) return hipSuccess;
    // A handful of messages: one atomic OR per bit.  More: rows built in LDS, provided a block of rows
    // fits (it always does within the shape limits of the interface).
    const int rmax = kStoreLdsBytes / (nw * 4);
    const bool rows = path == kStoreRows || (path == kStoreAuto && M >= kStoreRowsMinMessages);
    if (rows && rmax >= 1 && M <= 0x7FFFFFFF) {  // (queued message numbers are 32-bit)
        // About kStoreBlocks workgroups (one per compute unit): each scans the symbol column of its cluster
        // for all M messages, so fewer, larger ones scan less and more of them share the pair work.
        int R = (C * L + kStoreBlocks - 1) / kStoreBlocks;
        if (R > rmax) R = rmax;
        if (R > L) R = L;
        if (R < 1) R = 1;
        const int bpc = (L + R - 1) / R;
        const size_t lds = (size_t)R * nw * 4 + kStoreWaves * kStoreQueue * 4;
        if ((C & (C - 1)) == 0)
            hipLaunchKernelGGL(k_store_rows<true>, dim3((unsigned)(C * bpc)), dim3(kStoreThreads), lds, s, W, C, L, nw,
                               R, bpc, msgs, M, status);
        else
            hipLaunchKernelGGL(k_store_rows<false>, dim3((unsigned)(C * bpc)), dim3(kStoreThreads), lds, s, W, C, L,
                               nw, R, bpc, msgs, M, status);
        return hipGetLastError();
    }
    const int64_t total = M * C;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(k_store, dim3((unsigned)blocks), dim3(256), 0, s, W, C, L, nw, msgs, M, status);
    return hipGetLastError();
}

hipError_t launch_store_update(uint32_t *W, int C, int L, int nw, const int32_t *msgs, int64_t M, int32_t *status,
                               char *workspace, hipStream_t s)
{
    if (M == 0) return hipSuccess;
    const Geometry g = geometry(C, L);
    uint32_t *Wb = reinterpret_cast<uint32_t *>(workspace);
    uint32_t *has = reinterpret_cast<uint32_t *>(workspace + workspace_has_offset(C, L));
    uint64_t *full = reinterpret_cast<uint64_t *>(workspace + workspace_full_offset(C, L));
    uint32_t *hasc = g.padded ? reinterpret_cast<uint32_t *>(workspace + workspace_canonical_offset(C, L)) : nullptr;
    const int64_t total = M * C;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(k_store_update, dim3((unsigned)blocks), dim3(256), 0, s, W, Wb, has, hasc, C, L, nw, g.Lp, g.nwp,
                       msgs, M, status);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_summary_full, dim3(1), dim3(1024), 0, s, has, C, L, g.Lp, g.np, g.nwp, full);
    return hipGetLastError();
}

hipError_t launch_summary(const uint32_t *W, int C, int L, int nw, uint32_t *has, uint64_t *full, hipStream_t s)
{
    dim3 grid((unsigned)((nw + 63) / 64), (unsigned)C);
    hipLaunchKernelGGL(k_cluster_summary, grid, dim3(64 * kSumRows), 0, s, W, C, L, nw, has);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess || !full) return e;
    hipLaunchKernelGGL(k_summary_full, dim3(1), dim3(1024), 0, s, has, C, L, L, C * L, nw, full);
    return hipGetLastError();
}

hipError_t launch_prepare(const uint32_t *W, int C, int L, int nw, char *workspace, hipStream_t s)
{
    const Geometry g = geometry(C, L);
    uint32_t *Wb = reinterpret_cast<uint32_t *>(workspace);
    uint32_t *has = reinterpret_cast<uint32_t *>(workspace + workspace_has_offset(C, L));
    uint64_t *full = reinterpret_cast<uint64_t *>(workspace + workspace_full_offset(C, L));
    const int64_t words = (int64_t)g.np * g.nwp;
    int64_t blocks = (words + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    if (!g.padded) {
        const hipError_t e = launch_summary(W, C, L, nw, has, full, s);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k_fill_blocks, dim3((unsigned)blocks), dim3(256), 0, s, W, L, nw, words, Wb,
                           Wb + ((int64_t)g.np + C) * g.nwp);
        return hipGetLastError();
    }
    // padded: the table first, then its summaries from the table itself (a padded network in its own canonical
    // layout: clusters of Lp neurons), then the summaries in the interface's layout for the any-shape kernel
    hipLaunchKernelGGL(k_fill_padded, dim3((unsigned)blocks), dim3(256), 0, s, W, L, nw, g.Lp, g.nwp, words, Wb,
                       Wb + ((int64_t)g.np + C) * g.nwp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)((g.nwp + 63) / 64), (unsigned)C);
    hipLaunchKernelGGL(k_cluster_summary, grid, dim3(64 * kSumRows), 0, s, Wb, C, g.Lp, g.nwp, has);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_summary_full, dim3(1), dim3(1024), 0, s, has, C, L, g.Lp, g.np, g.nwp, full);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_summary(W, C, L, nw, reinterpret_cast<uint32_t *>(workspace + workspace_canonical_offset(C, L)), nullptr, s);
}

}  // namespace gbnn
