// Sparse form W' of the adjacency (Section IV-B, "Sparsification": only the nonzero elements and their
// coordinates) and sum-of-max retrieval (Eq. 6-7) from W' alone, for messages at the boundary.
//
// W' is one caller-owned buffer:
//   offsets  uint32[n + 1]   neighbours of neuron i are cols[offsets[i] .. offsets[i+1])
//   summary  uint32[C][nw]   bit i of row c: i is in c or has a neighbour in c (what a fully active
//                            cluster lets survive), followed by one uint64 of flags: row c is all ones
//   cols     uint16[...]     neuron numbers, ascending within a list; to the end of the buffer
// Retrieval: one wavefront per probe.  The activity vector lives in registers (word w in lane w % 64);
// a pass walks the clusters whose active set changed in the pass before (Lemma 1: the others cannot
// switch anything off).  A fully active cluster contributes its summary row.  The active neurons of the
// other clusters to walk are listed in LDS, and their neighbour lists are walked side by side: the 64
// lanes are split evenly among up to 64 listed neurons (64 lanes on one list, 32 on each of two, ... one
// lane per list), every lane reads eight list entries per load and ORs them into the bit vector T of the
// neuron's cluster in LDS (ds_or); then every neuron outside a walked cluster that is not in that
// cluster's T goes off.  A pass is thus a fixed, short chain of memory round trips (offsets, list chunks)
// whatever the number of active neurons.  The state and the number of passes are those of the kernels that
// read the packed W.
#include "gbnn_device.h"
#include "gbnn_internal.h"

namespace gbnn {
namespace {

constexpr int kSparseWaves = 4;                        // probes per workgroup

__device__ __forceinline__ uint32_t wave_sum(uint32_t x)
{
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) x += __shfl_xor(x, s, 64);
    return x;
}

// total = number of set bits of W: every thread strides over the words; one atomic add per workgroup
// (atomics on one address are served one after the other, so there are few workgroups).
__global__ __launch_bounds__(64) void k_sparse_zero(unsigned long long *total) { if (threadIdx.x == 0) *total = 0ull; }
__global__ __launch_bounds__(1024) void k_sparse_total(const uint32_t *__restrict__ W, int64_t words,
                                                       unsigned long long *total)
{
    __shared__ uint32_t part[16];
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    uint32_t pc = 0;  // at most 32 * words / stride per thread: no overflow within the shape limits
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < words; t += stride) pc += __popc(W[t]);
    pc = wave_sum(pc);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = pc;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long sum = 0;
        for (int i = 0; i < 16; ++i) sum += part[i];
        if (sum) atomicAdd(total, sum);
    }
}

// offsets[i + 1] = degree of neuron i (offsets[0] = 0); one wave per row.
__global__ __launch_bounds__(256) void k_sparse_degree(const uint32_t *__restrict__ W, int n, int nw,
                                                       uint32_t *__restrict__ offsets)
{
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= n) return;
    uint32_t pc = 0;
    for (int w = lane; w < nw; w += 64) pc += __popc(W[(int64_t)i * nw + w]);
    pc = wave_sum(pc);
    if (lane == 0) {
        offsets[i + 1] = pc;
        if (i == 0) offsets[0] = 0u;
    }
}

// In-place inclusive scan of offsets[1..n] by one workgroup: every thread sums a run of consecutive
// entries, the run totals are scanned in LDS, then every thread rewrites its run.
__global__ __launch_bounds__(1024) void k_sparse_scan(uint32_t *__restrict__ offsets, int n, uint32_t capacity,
                                                      int32_t *__restrict__ status)
{
    __shared__ uint32_t part[1024];
    const int run = (n + 1023) / 1024;
    const int lo = threadIdx.x * run;
    const int hi = lo + run < n ? lo + run : n;
    uint32_t sum = 0;
    for (int i = lo; i < hi; ++i) sum += offsets[i + 1];
    part[threadIdx.x] = sum;
    __syncthreads();
    for (int s = 1; s < 1024; s <<= 1) {
        const uint32_t add = threadIdx.x >= (unsigned)s ? part[threadIdx.x - s] : 0u;
        __syncthreads();
        part[threadIdx.x] += add;
        __syncthreads();
    }
    uint32_t acc = part[threadIdx.x] - sum;
    for (int i = lo; i < hi; ++i) {
        acc += offsets[i + 1];
        offsets[i + 1] = acc;
    }
    if (threadIdx.x == 1023 && part[1023] > capacity && status) atomicOr(status, 1);
}

// cols[offsets[i] ..] = the set bits of row i, ascending; one wave per row, 64 words at a time.  Entries
// beyond the capacity of the buffer are not written (the scan has reported that case).
__global__ __launch_bounds__(256) void k_sparse_fill(const uint32_t *__restrict__ W, int n, int nw,
                                                     const uint32_t *__restrict__ offsets,
                                                     uint16_t *__restrict__ cols, uint32_t capacity)
{
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= n) return;
    uint32_t at = offsets[i];
    for (int w0 = 0; w0 < nw; w0 += 64) {
        const int w = w0 + lane;
        uint32_t word = w < nw ? W[(int64_t)i * nw + w] : 0u;
        const uint32_t pc = __popc(word);
        uint32_t before = pc;  // inclusive prefix sum over the lanes
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
            const uint32_t up = __shfl_up(before, s, 64);
            if (lane >= s) before += up;
        }
        const uint32_t total = __shfl(before, 63, 64);
        uint32_t pos = at + before - pc;
        while (word) {
            const int b = __builtin_ctz(word);
            word &= word - 1u;
            if (pos < capacity) cols[pos] = (uint16_t)(w * 32 + b);
            ++pos;
        }
        at += total;
    }
}

struct SparseArgs {
    const uint32_t *offsets;
    const uint32_t *summary;
    const uint64_t *full;
    const uint16_t *cols;
    uint32_t capacity;
    const int32_t *sym_in;
    uint32_t *bits_out;
    int32_t *sym_out;
    int32_t *iters;
    int64_t K;
    int C, L, n, nw, wpc;  // wpc = L / 32 words per cluster
    int group;             // clusters whose bit vectors T fit a wave's LDS at once
    int wave_words;        // LDS words per wave
    int max_iters;
};

constexpr int kSparseList = 128;  // neurons listed at a time

// LDS of one wave: cur[nw] (the final vector, for the symbols), nlist[kSparseList],
// T[group][nw].
__host__ __device__ inline int sparse_wave_words(int nw, int group) { return nw + kSparseList + group * nw; }

// NS = words of the activity vector per lane (1, 2, 4 or 8: nw <= 64 NS).
template <int NS>
__global__ __launch_bounds__(64 * kSparseWaves) __attribute__((amdgpu_waves_per_eu(NS == 8 ? 4 : NS == 4 ? 6 : 8))) void
k_retrieve_sparse(SparseArgs a)
{
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t k = (int64_t)blockIdx.x * kSparseWaves + wave;
    if (k >= a.K) return;  // the whole wave
    const int nw = a.nw, wpc = a.wpc, C = a.C, L = a.L;
    uint32_t *cur = lds + wave * a.wave_words;
    uint32_t *nlist = cur + nw;
    uint32_t *T = nlist + kSparseList;
    const uint64_t summary_full = *a.full;

    // word w = lane + 64 u of the activity vector; its cluster; Section III-C: an erased cluster starts
    // with all of its neurons on, a known one with the neuron of its symbol
    uint32_t v[NS], d[NS], acc[NS];
    int cl[NS];
#pragma unroll
    for (int u = 0; u < NS; ++u) {
        const int w = lane + 64 * u;
        cl[u] = w < nw ? w / wpc : -1;
        v[u] = 0u;
        d[u] = 0u;
        if (w < nw) {
            const int32_t s = a.sym_in[k * C + cl[u]];
            const int wi = w - cl[u] * wpc;
            v[u] = (uint32_t)s < (uint32_t)L ? ((s >> 5) == wi ? 1u << (s & 31) : 0u) : 0xFFFFFFFFu;
        }
    }

    int32_t iters = 0;
    for (int p = 1;; ++p) {
        // per cluster: number of active neurons, and whether any changed in the pass before
        uint64_t emptym, fullm, srcm;
        if (p == 1) {
            // as the probe arrives: a known cluster holds one neuron, an erased one all of its L >= 32
            const bool erased = lane < C && (uint32_t)a.sym_in[k * C + lane] >= (uint32_t)L;
            emptym = 0;
            fullm = ballot(erased);
            srcm = ballot(lane < C);
        } else {
            // every lane adds what its words hold to the slots of their clusters (T[0 .. C) and T[C .. 2C))
            if (lane < C) {
                T[lane] = 0u;
                T[C + lane] = 0u;
            }
            wave_lds_sync();
#pragma unroll
            for (int u = 0; u < NS; ++u) {
                if (cl[u] >= 0 && v[u]) atomicAdd(&T[cl[u]], (uint32_t)__popc(v[u]));
                if (cl[u] >= 0 && d[u]) atomicOr(&T[C + cl[u]], 1u);
            }
            wave_lds_sync();
            const uint32_t cnt = lane < C ? T[lane] : 0u, chg = lane < C ? T[C + lane] : 0u;
            emptym = ballot(lane < C && cnt == 0u);
            fullm = ballot(lane < C && cnt == (uint32_t)L);
            srcm = ballot(lane < C && chg != 0u);
            wave_lds_sync();
        }
#pragma unroll
        for (int u = 0; u < NS; ++u) acc[u] = emptym ? 0u : v[u];
        if (emptym) srcm = 0;  // a cluster without an active neuron: nobody reaches C - 1 clusters
        // fully active clusters: their summary rows (one that is all ones changes nothing)
        for (uint64_t fm = srcm & fullm & ~summary_full; fm; fm &= fm - 1ull) {
            const int c = __builtin_ctzll(fm);
#pragma unroll
            for (int u = 0; u < NS; ++u) {
                const int w = lane + 64 * u;
                if (w < nw) acc[u] &= a.summary[(int64_t)c * nw + w];
            }
        }
        // the other clusters to walk, as many at a time as have their bit vectors T in LDS together
        uint64_t walk = srcm & ~fullm;
        while (walk) {
            uint64_t grp = walk;
            int ng = __builtin_popcountll(grp);
            if (ng > a.group) {  // more clusters than bit vectors: the lowest a.group of them now
                grp = 0;
                for (int g = 0; g < a.group; ++g) {
                    grp |= walk & (0ull - walk);
                    walk &= walk - 1ull;
                }
                ng = a.group;
            } else {
                walk = 0;
            }
            for (int i = lane; i < ng * nw; i += 64) T[i] = 0u;
            // the active neurons of these clusters, and for each the row of T its list goes to
            uint32_t pw[NS], trow[NS];
#pragma unroll
            for (int u = 0; u < NS; ++u) {
                const bool in = cl[u] >= 0 && ((grp >> cl[u]) & 1ull);
                pw[u] = in ? v[u] : 0u;
                trow[u] = in ? (uint32_t)__builtin_popcountll(grp & ((1ull << cl[u]) - 1ull)) : 0u;
            }
            for (;;) {
                // list up to kSparseList of them: entry = (row of T) << 16 | neuron.  The position of a lane's
                // first bit = the bits in lower lanes = sum over r of #(lower lanes with more than r bits).
                uint32_t base = 0;
                bool left = false;
#pragma unroll
                for (int u = 0; u < NS; ++u) {
                    const uint32_t pc = __popc(pw[u]);
                    uint64_t mk = ballot(pc > 0u);
                    if (!mk) continue;
                    uint32_t pos = base;
                    for (uint32_t r = 1; mk; ++r) {
                        pos += mbcnt(mk);
                        base += (uint32_t)__builtin_popcountll(mk);
                        mk = ballot(pc > r);
                    }
                    while (pw[u] && pos < (uint32_t)kSparseList) {
                        const int b = __builtin_ctz(pw[u]);
                        pw[u] &= pw[u] - 1u;
                        nlist[pos++] = (trow[u] << 16) | (uint32_t)((lane + 64 * u) * 32 + b);
                    }
                    left = left || pw[u] != 0u;
                }
                const int listed = base < (uint32_t)kSparseList ? (int)base : kSparseList;
                wave_lds_sync();
                // walk the lists, up to 64 neurons side by side, P lanes on each
                for (int n0 = 0; n0 < listed; n0 += 64) {
                    const int here = listed - n0 < 64 ? listed - n0 : 64;
                    int lgp = 6;  // P = 2^lgp lanes per list: 64 for one neuron, 32 for two, ..., 1 for 33 to 64
                    while ((here << lgp) > 64) --lgp;
                    const int ni = lane >> lgp, sub = lane & ((1 << lgp) - 1);
                    if (ni < here) {
                        const uint32_t ent = nlist[n0 + ni];
                        const uint32_t j = ent & 0xFFFFu;
                        uint32_t *Tr = T + (ent >> 16) * nw;
                        uint32_t end = a.offsets[j + 1];
                        end = end < a.capacity ? end : a.capacity;
                        uint32_t beg = a.offsets[j];
                        beg = beg < end ? beg : end;
                        // aligned chunks of eight entries; two loads in flight per lane
                        const uint32_t step = 8u << lgp;
                        for (uint32_t t0 = (beg & ~7u) + 8u * (uint32_t)sub; t0 < end; t0 += 2u * step) {
                            uint4 ch[2];
#pragma unroll
                            for (int q = 0; q < 2; ++q) {
                                const uint32_t t = t0 + q * step;
                                ch[q] = t < end ? *reinterpret_cast<const uint4 *>(a.cols + t) : make_uint4(0, 0, 0, 0);
                            }
#pragma unroll
                            for (int q = 0; q < 2; ++q) {
                                const uint32_t t = t0 + q * step;
                                if (q == 1 && t >= end) break;  // (short lists: most lanes have one chunk)
                                // entries t .. t + 7, of which [beg, end) belong to the list
                                const uint32_t lo = beg > t ? beg - t : 0u, hi = end - t < 8u ? end - t : 8u;
                                const uint32_t live = (0xFFu >> (8u - hi)) & (0xFFu << lo);
                                const uint32_t wd[4] = {ch[q].x, ch[q].y, ch[q].z, ch[q].w};
#pragma unroll
                                for (int e = 0; e < 8; ++e) {
                                    const uint32_t col = (e & 1) ? wd[e >> 1] >> 16 : wd[e >> 1] & 0xFFFFu;
                                    if (((live >> e) & 1u) && col < (uint32_t)a.n) atomicOr(&Tr[col >> 5], 1u << (col & 31u));
                                }
                            }
                        }
                    }
                }
                wave_lds_sync();
                if (!ballot(left)) break;
            }
            // every neuron outside a walked cluster that is not in that cluster's T goes off
            int row = 0;
            for (uint64_t g = grp; g; g &= g - 1ull, ++row) {
                const int c = __builtin_ctzll(g);
#pragma unroll
                for (int u = 0; u < NS; ++u) {
                    const int w = lane + 64 * u;
                    if (w < nw && cl[u] != c) acc[u] &= T[row * nw + w];
                }
            }
            wave_lds_sync();
        }
        bool changed = false;
#pragma unroll
        for (int u = 0; u < NS; ++u) {
            d[u] = acc[u] ^ v[u];
            changed = changed || d[u] != 0u;
            v[u] = acc[u];
        }
        const bool any = ballot(changed) != 0ull;
        if (!any) {
            iters = p;
            break;
        }
        if (p == a.max_iters) {
            iters = -p;
            break;
        }
    }

    if (a.iters && lane == 0) a.iters[k] = iters;
    if (a.bits_out) {
#pragma unroll
        for (int u = 0; u < NS; ++u) {
            const int w = lane + 64 * u;
            if (w < nw) a.bits_out[k * nw + w] = v[u];
        }
    }
    if (a.sym_out) {
#pragma unroll
        for (int u = 0; u < NS; ++u) {
            const int w = lane + 64 * u;
            if (w < nw) cur[w] = v[u];
        }
        wave_lds_sync();
        if (lane < C) {
            uint32_t cnt = 0;
            int32_t pos = 0;
            for (int i = 0; i < wpc; ++i) {
                const uint32_t word = cur[lane * wpc + i];
                if (word && !cnt) pos = i * 32 + __builtin_ctz(word);
                cnt += __popc(word);
            }
            a.sym_out[k * C + lane] = cnt == 1u ? pos : (cnt == 0u ? GBNN_SYM_NONE : GBNN_SYM_AMBIGUOUS);
        }
    }
}

}  // namespace

size_t sparse_summary_offset(int n) { return (((size_t)n + 1) * sizeof(uint32_t) + 255) & ~(size_t)255; }
size_t sparse_full_offset(int C, int n, int nw)
{
    return sparse_summary_offset(n) + (((size_t)C * nw * sizeof(uint32_t) + 255) & ~(size_t)255);
}
size_t sparse_cols_offset(int C, int n, int nw) { return sparse_full_offset(C, n, nw) + 256; }

// Entries of cols[] a buffer of Wp_bytes has room for: whole 16-byte pieces only (retrieval reads the lists
// eight entries at a time), the same figure for filling and for reading.
static uint32_t sparse_capacity(size_t Wp_bytes, int C, int n, int nw)
{
    const size_t room = ((Wp_bytes - sparse_cols_offset(C, n, nw)) & ~(size_t)15) / sizeof(uint16_t);
    return room > 0xFFFFFFF8ull ? 0xFFFFFFF8u : (uint32_t)room;
}

hipError_t launch_sparse_count(const uint32_t *W, int n, int nw, unsigned long long *total, hipStream_t s)
{
    hipLaunchKernelGGL(k_sparse_zero, dim3(1), dim3(64), 0, s, total);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t words = (int64_t)n * nw;
    int64_t blocks = (words + 1023) / 1024;
    if (blocks > 64) blocks = 64;
    hipLaunchKernelGGL(k_sparse_total, dim3((unsigned)blocks), dim3(1024), 0, s, W, words, total);
    return hipGetLastError();
}

hipError_t launch_sparsify(const uint32_t *W, int C, int L, int nw, char *Wp, size_t Wp_bytes, int32_t *status,
                           hipStream_t s)
{
    const int n = C * L;
    uint32_t *offsets = reinterpret_cast<uint32_t *>(Wp);
    uint32_t *summary = reinterpret_cast<uint32_t *>(Wp + sparse_summary_offset(n));
    uint64_t *full = reinterpret_cast<uint64_t *>(Wp + sparse_full_offset(C, n, nw));
    uint16_t *cols = reinterpret_cast<uint16_t *>(Wp + sparse_cols_offset(C, n, nw));
    const uint32_t capacity = sparse_capacity(Wp_bytes, C, n, nw);
    const dim3 rows((unsigned)((n + 3) / 4));
    hipLaunchKernelGGL(k_sparse_degree, rows, dim3(256), 0, s, W, n, nw, offsets);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_sparse_scan, dim3(1), dim3(1024), 0, s, offsets, n, capacity, status);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_sparse_fill, rows, dim3(256), 0, s, W, n, nw, offsets, cols, capacity);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_summary(W, C, L, nw, summary, full, s);
}

hipError_t launch_retrieve_sparse(const char *Wp, size_t Wp_bytes, int C, int L, int nw, const int32_t *probes,
                                  int64_t K, int max_iters, uint32_t *bits_out, int32_t *sym_out, int32_t *iters,
                                  hipStream_t s)
{
    if (K == 0) return hipSuccess;
    const int n = C * L;
    SparseArgs a{};
    a.offsets = reinterpret_cast<const uint32_t *>(Wp);
    a.summary = reinterpret_cast<const uint32_t *>(Wp + sparse_summary_offset(n));
    a.full = reinterpret_cast<const uint64_t *>(Wp + sparse_full_offset(C, n, nw));
    a.cols = reinterpret_cast<const uint16_t *>(Wp + sparse_cols_offset(C, n, nw));
    a.capacity = sparse_capacity(Wp_bytes, C, n, nw);
    a.sym_in = probes;
    a.bits_out = bits_out;
    a.sym_out = sym_out;
    a.iters = iters;
    a.K = K;
    a.C = C;
    a.L = L;
    a.n = n;
    a.nw = nw;
    a.wpc = L / 32;
    a.max_iters = max_iters;
    // LDS per wave: about 10 KiB at most (so that a compute unit keeps four 4-wave workgroups), less for
    // small networks; the bit vectors of `group` clusters fit at once
    int group = (2560 - kSparseList - nw) / nw;
    if (group > C) group = C;
    if (group < 1) group = 1;
    a.group = group;
    a.wave_words = sparse_wave_words(nw, group);
    const size_t lds = (size_t)a.wave_words * kSparseWaves * sizeof(uint32_t);
    const int64_t blocks = (K + kSparseWaves - 1) / kSparseWaves;
    const dim3 grid((unsigned)blocks), block(64 * kSparseWaves);
    if (nw <= 64)
        hipLaunchKernelGGL(k_retrieve_sparse<1>, grid, block, lds, s, a);
    else if (nw <= 128)
        hipLaunchKernelGGL(k_retrieve_sparse<2>, grid, block, lds, s, a);
    else if (nw <= 256)
        hipLaunchKernelGGL(k_retrieve_sparse<4>, grid, block, lds, s, a);
    else
        hipLaunchKernelGGL(k_retrieve_sparse<8>, grid, block, lds, s, a);
    return hipGetLastError();
}

}  // namespace gbnn
