// Any-shape retrieval: one wavefront (= one 64-thread workgroup) per probe, the probe's packed
// activity and the bit-sliced scores live in LDS.  Clusters need not be aligned to 32-bit words
// (L = 3, L = 16, ...): every cluster operation goes through own_mask(), the bits of a word
// that belong to a cluster.  Lane l owns words l, l+64, ... of every LDS array, so the only
// cross-lane traffic is the wave-uniform read of activity words and the barriers around it.
// Same rule definitions as the one-wave-per-probe register kernel; this one favours plainness.
#include "gbnn_device.h"
#include "gbnn_internal.h"

namespace gbnn {
namespace {

__device__ __forceinline__ int wave_sum(int x)
{
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

__device__ __forceinline__ uint32_t uniform(uint32_t x) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)x); }

struct G {
    const RetrieveArgs &a;
    int lane;
    uint32_t *v, *acc, *R, *aux, *pl;  // LDS: [nw] each, pl is [kPlanes][nw]

    __device__ int first_word(int c) const { return (c * a.L) >> 5; }
    __device__ int last_word(int c) const { return ((c + 1) * a.L - 1) >> 5; }

    __device__ int cluster_count(int c) const
    {
        int cnt = 0;
        for (int w = first_word(c) + lane; w <= last_word(c); w += 64) cnt += __popc(v[w] & own_mask(c, a.L, w));
        return wave_sum(cnt);
    }

    // acc = v AND over all clusters c' of (signals from c' | own-cluster mask of c').
    __device__ void som_pass() const
    {
        for (int w = lane; w < a.nw; w += 64) acc[w] = v[w];
        for (int c = 0; c < a.C; ++c) {
            const int cnt = cluster_count(c);
            for (int w = lane; w < a.nw; w += 64) R[w] = own_mask(c, a.L, w);
            if (cnt == a.L) {
                const uint32_t *row = a.hasc + (int64_t)c * a.nw;
                for (int w = lane; w < a.nw; w += 64) R[w] |= row[w];
            } else if (cnt > 0) {
                for (int ww = first_word(c); ww <= last_word(c); ++ww) {
                    uint32_t word = uniform(v[ww] & own_mask(c, a.L, ww));
                    while (word) {
                        const int j = 32 * ww + __builtin_ctz(word);
                        word &= word - 1;
                        const uint32_t *row = a.W + (int64_t)j * a.nw;
                        for (int w = lane; w < a.nw; w += 64) R[w] |= row[w];
                    }
                }
            }
            for (int w = lane; w < a.nw; w += 64) acc[w] &= R[w];
        }
    }

    // Bit-sliced sum of the rows of all active neurons; returns their number.
    __device__ int count_signals() const
    {
        for (int q = 0; q < kPlanes; ++q)
            for (int w = lane; w < a.nw; w += 64) pl[q * a.nw + w] = 0u;
        int rows = 0;
        for (int ww = 0; ww < a.nw; ++ww) {
            uint32_t word = uniform(v[ww]);
            while (word) {
                const int j = 32 * ww + __builtin_ctz(word);
                word &= word - 1;
                ++rows;
                const int np = 32 - __builtin_clz((unsigned)rows);
                const uint32_t *row = a.W + (int64_t)j * a.nw;
                for (int w = lane; w < a.nw; w += 64) {
                    uint32_t carry = row[w];
                    for (int q = 0; q < np; ++q) {
                        const uint32_t d = pl[q * a.nw + w];
                        pl[q * a.nw + w] = d ^ carry;
                        carry &= d;
                    }
                }
            }
        }
        return rows;
    }

    // v_next (in acc) from Eq. (3)-(5) given the counters of the current v.
    __device__ void sos_select(int rows) const
    {
        const unsigned top = (unsigned)(rows + a.gamma);
        const int P = top ? 32 - __builtin_clz(top) : 0;
        if (a.gamma) {
            for (int w = lane; w < a.nw; w += 64) {
                uint32_t cy = 0u;
                for (int q = 0; q < P; ++q) {
                    const uint32_t g = ((a.gamma >> q) & 1) ? v[w] : 0u;
                    const uint32_t d = pl[q * a.nw + w];
                    pl[q * a.nw + w] = d ^ g ^ cy;
                    cy = (d & g) | (cy & (d ^ g));
                }
            }
        }
        for (int w = lane; w < a.nw; w += 64) acc[w] = 0u;
        for (int c = 0; c < a.C; ++c) {
            const int wb = first_word(c), we = last_word(c);
            // every loop below is over the words this lane owns (w % 64 == lane)
            const int w0 = wb + ((lane - wb) & 63);
            for (int w = w0; w <= we; w += 64) aux[w] = own_mask(c, a.L, w);
            for (int q = P - 1; q >= 0; --q) {
                bool mine = false;
                for (int w = w0; w <= we; w += 64) mine = mine || ((aux[w] & pl[q * a.nw + w]) != 0u);
                if (__any(mine))
                    for (int w = w0; w <= we; w += 64) aux[w] &= pl[q * a.nw + w];
            }
            for (int w = w0; w <= we; w += 64) acc[w] |= aux[w];
        }
    }

    __device__ bool commit() const  // v <- acc; returns whether anything changed
    {
        bool diff = false;
        for (int w = lane; w < a.nw; w += 64) {
            diff = diff || (acc[w] != v[w]);
        }
        const bool changed = __any(diff);
        __syncthreads();
        for (int w = lane; w < a.nw; w += 64) v[w] = acc[w];
        __syncthreads();
        return changed;
    }
};

__global__ __launch_bounds__(64) void k_retrieve_generic(RetrieveArgs a)
{
    extern __shared__ uint32_t sm[];
    G g{a, (int)threadIdx.x, sm, sm + a.nw, sm + 2 * a.nw, sm + 3 * a.nw, sm + 4 * a.nw};
    const int lane = g.lane;

    for (int64_t k = blockIdx.x; k < a.K; k += gridDim.x) {
        if (a.sym_in) {
            // the message boundary: one symbol per cluster, anything outside [0, L) = erased (Section II-A)
            for (int w = lane; w < a.nw; w += 64) g.v[w] = 0u;
            __syncthreads();
            for (int c = lane; c < a.C; c += 64) {
                const int32_t sy = a.sym_in[k * a.C + c];
                if (sy >= 0 && sy < a.L) {
                    const int i = c * a.L + sy;
                    atomicOr(&g.v[i >> 5], 1u << (i & 31));  // clusters may share a word
                }
            }
        } else {
            const uint8_t *src = a.V0 + k * a.n;
            for (int w = lane; w < a.nw; w += 64) {
                uint32_t word = 0u;
                for (int b = 0; b < 32; ++b) {
                    const int i = 32 * w + b;
                    if (i < a.n) word |= (uint32_t)(src[i] & 1u) << b;
                }
                g.v[w] = word;
            }
        }
        __syncthreads();

        int it = 0;
        if (a.rule == GBNN_SUM_OF_MAX) {
            for (int c = 0; c < a.C; ++c) {  // erased clusters start fully active
                if (g.cluster_count(c) == 0)
                    for (int w = lane; w < a.nw; w += 64) g.v[w] |= own_mask(c, a.L, w);
                __syncthreads();
            }
            int p = 0;
            for (;;) {
                g.som_pass();
                ++p;
                const bool changed = g.commit();
                if (!changed) { it = p; break; }
                if (p == a.max_iters) { it = -p; break; }
            }
        } else if (a.rule == GBNN_HYBRID) {
            uint32_t *er = g.aux;  // bits of erased clusters
            for (int w = lane; w < a.nw; w += 64) er[w] = 0u;
            int known = 0;
            for (int c = 0; c < a.C; ++c) {
                if (g.cluster_count(c) == 0) {
                    for (int w = lane; w < a.nw; w += 64) er[w] |= own_mask(c, a.L, w);
                } else {
                    ++known;
                }
            }
            const int rows = g.count_signals();
            const int np = rows ? 32 - __builtin_clz((unsigned)rows) : 0;
            for (int w = lane; w < a.nw; w += 64) {
                uint32_t eq = 0xFFFFFFFFu;
                for (int q = 0; q < np; ++q) eq &= ((known >> q) & 1) ? g.pl[q * a.nw + w] : ~g.pl[q * a.nw + w];
                g.acc[w] = (eq & er[w]) | (g.v[w] & ~er[w]);
            }
            g.commit();
            int p = 1;
            if (p == a.max_iters) {
                it = -p;
            } else {
                for (;;) {
                    g.som_pass();
                    for (int w = lane; w < a.nw; w += 64) g.acc[w] = (g.acc[w] & er[w]) | (g.v[w] & ~er[w]);
                    ++p;
                    const bool changed = g.commit();
                    if (!changed) { it = p; break; }
                    if (p == a.max_iters) { it = -p; break; }
                }
            }
        } else {
            int p = 0;
            for (;;) {
                const int rows = g.count_signals();
                g.sos_select(rows);
                ++p;
                const bool changed = g.commit();
                if (!changed) { it = p; break; }
                if (p == a.max_iters) { it = -p; break; }
            }
        }

        if (a.iters && lane == 0) a.iters[k] = it;
        if (a.sym_in) {
            if (a.bits_out)
                for (int w = lane; w < a.nw; w += 64) a.bits_out[k * a.nw + w] = g.v[w];
            if (a.sym_out) {
                // the symbol of a cluster: its active neuron if it has exactly one, -1 none, -2 several
                for (int c = lane; c < a.C; c += 64) {
                    int cnt = 0, pos = 0;
                    for (int w = g.first_word(c); w <= g.last_word(c); ++w) {
                        const uint32_t m = g.v[w] & own_mask(c, a.L, w);
                        if (m) pos = 32 * w + __builtin_ctz(m) - c * a.L;
                        cnt += __popc(m);
                    }
                    a.sym_out[k * a.C + c] = cnt == 1 ? pos : (cnt == 0 ? -1 : -2);
                }
            }
        } else {
            uint8_t *dst = a.Vout + k * a.n;
            for (int w = lane; w < a.nw; w += 64) {
                const uint32_t word = g.v[w];
                for (int b = 0; b < 32; ++b) {
                    const int i = 32 * w + b;
                    if (i < a.n) dst[i] = (uint8_t)((word >> b) & 1u);
                }
            }
        }
        __syncthreads();
    }
}

}  // namespace

hipError_t launch_retrieve_generic(const RetrieveArgs &a, hipStream_t s)
{
    if (a.K == 0) return hipSuccess;
    int64_t blocks = a.K;
    const int64_t cap = 256 * 16;
    if (blocks > cap) blocks = cap;
    const size_t lds = (size_t)(4 + kPlanes) * (size_t)a.nw * sizeof(uint32_t);
    hipLaunchKernelGGL(k_retrieve_generic, dim3((unsigned)blocks), dim3(64), lds, s, a);
    return hipGetLastError();
}

}  // namespace gbnn
