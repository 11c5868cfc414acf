// Any-shape retrieval: one wavefront (= one 64-thread workgroup) per probe, the probe's packed
// activity lives in LDS, the bit-sliced scores in registers.  Clusters need not be aligned to 32-bit words
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

constexpr int kPerLane = GBNN_MAX_N / 32 / 64;  // words of a packed vector per lane

struct G {
    const RetrieveArgs &a;
    int lane;
    uint32_t *v, *acc, *aux;  // LDS: [nw] each

    // lane l owns the words l, l + 64, ...: at most kPerLane of them
    __device__ int word_of(int t) const { return lane + 64 * t; }
    __device__ bool mine(int t) const { return lane + 64 * t < a.nw; }

    __device__ int first_word(int c) const { return (c * a.L) >> 5; }
    __device__ int last_word(int c) const { return ((c + 1) * a.L - 1) >> 5; }

    __device__ int cluster_count(int c) const
    {
        int cnt = 0;
        for (int w = first_word(c) + lane; w <= last_word(c); w += 64) cnt += __popc(v[w] & own_mask(c, a.L, w));
        return wave_sum(cnt);
    }

    // acc = v AND over all clusters c' of (signals from c' | own-cluster mask of c').  A lane's words of acc
    // and of the signals stay in registers (at most kPerLane of them); rows are fetched four at a time.
    __device__ void som_pass() const
    {
        uint32_t accr[kPerLane];
#pragma unroll
        for (int t = 0; t < kPerLane; ++t) accr[t] = mine(t) ? v[word_of(t)] : 0u;
        for (int c = 0; c < a.C; ++c) {
            const int cnt = cluster_count(c);
            if (cnt == 0) {  // nobody signals from an empty cluster: only its own (empty) neurons would stay
#pragma unroll
                for (int t = 0; t < kPerLane; ++t) accr[t] &= mine(t) ? own_mask(c, a.L, word_of(t)) : 0u;
                continue;
            }
            uint32_t Rr[kPerLane];
#pragma unroll
            for (int t = 0; t < kPerLane; ++t) Rr[t] = mine(t) ? own_mask(c, a.L, word_of(t)) : 0u;
            if (cnt == a.L) {
                const uint32_t *row = a.hasc + (int64_t)c * a.nw;
#pragma unroll
                for (int t = 0; t < kPerLane; ++t)
                    if (mine(t)) Rr[t] |= row[word_of(t)];
            } else {
                // the words of the cluster that hold an active neuron, found by a ballot over their owners
                const int fw = first_word(c), lw = last_word(c);
#pragma unroll 1
                for (int s = 0; s < kPerLane; ++s) {
                    if (64 * s + 63 < fw || 64 * s > lw) continue;
                    const uint32_t held = mine(s) ? v[word_of(s)] & own_mask(c, a.L, word_of(s)) : 0u;
                    uint64_t holders = ballot(held != 0u);
                    while (holders) {
                        const int src = __builtin_ctzll(holders);
                        holders &= holders - 1ull;
                        uint32_t word = readlane(held, src);
                        const int base = 32 * (src + 64 * s);
                        while (word) {
                            const uint32_t *row[4];
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                if (word || q == 0) {
                                    row[q] = a.W + (int64_t)(base + __builtin_ctz(word)) * a.nw;
                                    word &= word - 1;
                                } else {
                                    row[q] = row[q - 1];  // (the same row again: harmless under OR)
                                }
                            }
                            uint32_t r[4][kPerLane];
#pragma unroll
                            for (int q = 0; q < 4; ++q)
#pragma unroll
                                for (int t = 0; t < kPerLane; ++t) r[q][t] = mine(t) ? row[q][word_of(t)] : 0u;
#pragma unroll
                            for (int q = 0; q < 4; ++q)
#pragma unroll
                                for (int t = 0; t < kPerLane; ++t) Rr[t] |= r[q][t];
                        }
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < kPerLane; ++t) accr[t] &= Rr[t];
        }
#pragma unroll
        for (int t = 0; t < kPerLane; ++t)
            if (mine(t)) acc[word_of(t)] = accr[t];
    }

    // Bit-sliced sum of the rows of all active neurons (digit q of the count of neuron 32 w + b = bit b of
    // pl[q][t], w the lane's t-th word); returns their number.  The digits live in registers: every loop over
    // them is unrolled, the number of digits in use is the same for all lanes.  NP digits are kept; a count
    // that needs more sets the neuron's bit in ovf (its digits are then meaningless).
    template <int NP>
    __device__ int count_signals(uint32_t (&pl)[NP][kPerLane], uint32_t (&ovf)[kPerLane]) const
    {
#pragma unroll
        for (int t = 0; t < kPerLane; ++t) ovf[t] = 0u;
#pragma unroll
        for (int q = 0; q < NP; ++q)
#pragma unroll
            for (int t = 0; t < kPerLane; ++t) pl[q][t] = 0u;
        int rows = 0;
#pragma unroll 1
        for (int s = 0; s < kPerLane; ++s) {
            if (64 * s >= a.nw) continue;
            const uint32_t held = mine(s) ? v[word_of(s)] : 0u;
            uint64_t holders = ballot(held != 0u);  // the words that hold an active neuron, by owner
            while (holders) {
                const int src = __builtin_ctzll(holders);
                holders &= holders - 1ull;
                uint32_t word = readlane(held, src);
                const int base = 32 * (src + 64 * s);
                while (word) {
                    // two rows fetched together, added one after the other
                    const uint32_t *row[2];
                    row[0] = a.W + (int64_t)(base + __builtin_ctz(word)) * a.nw;
                    word &= word - 1;
                    const bool two = word != 0u;
                    row[1] = row[0];
                    if (two) {
                        row[1] = a.W + (int64_t)(base + __builtin_ctz(word)) * a.nw;
                        word &= word - 1;
                    }
                    uint32_t r[2][kPerLane];
#pragma unroll
                    for (int q = 0; q < 2; ++q)
#pragma unroll
                        for (int t = 0; t < kPerLane; ++t) r[q][t] = mine(t) ? row[q][word_of(t)] : 0u;
                    rows += two ? 2 : 1;
                    const int np = 32 - __builtin_clz((unsigned)rows);  // digits of the largest count so far
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        if (h == 1 && !two) break;
#pragma unroll
                        for (int q = 0; q < NP; ++q) {
                            if (q < np) {
#pragma unroll
                                for (int t = 0; t < kPerLane; ++t) {
                                    const uint32_t d = pl[q][t];
                                    pl[q][t] = d ^ r[h][t];
                                    r[h][t] &= d;
                                }
                            }
                        }
#pragma unroll
                        for (int t = 0; t < kPerLane; ++t) ovf[t] |= r[h][t];  // carry out of the last digit kept
                    }
                }
            }
        }
        return rows;
    }

    // v_next (in acc) from Eq. (3)-(5) given the counters of the current v.
    __device__ void sos_select(int rows, uint32_t (&pl)[kPlanes][kPerLane]) const
    {
        const unsigned top = (unsigned)(rows + a.gamma);
        const int P = top ? 32 - __builtin_clz(top) : 0;
        if (a.gamma) {
            uint32_t cy[kPerLane], vv[kPerLane];
#pragma unroll
            for (int t = 0; t < kPerLane; ++t) {
                cy[t] = 0u;
                vv[t] = mine(t) ? v[word_of(t)] : 0u;
            }
#pragma unroll
            for (int q = 0; q < kPlanes; ++q) {
                if (q < P) {
                    const bool bit = (a.gamma >> q) & 1;
#pragma unroll
                    for (int t = 0; t < kPerLane; ++t) {
                        const uint32_t g = bit ? vv[t] : 0u;
                        const uint32_t d = pl[q][t];
                        pl[q][t] = d ^ g ^ cy[t];
                        cy[t] = (d & g) | (cy[t] & (d ^ g));
                    }
                }
            }
        }
        uint32_t next[kPerLane];
#pragma unroll
        for (int t = 0; t < kPerLane; ++t) next[t] = 0u;
        for (int c = 0; c < a.C; ++c) {
            // the neurons of the cluster whose count is the cluster's maximum: digit by digit from the top
            uint32_t m[kPerLane];
#pragma unroll
            for (int t = 0; t < kPerLane; ++t) m[t] = mine(t) ? own_mask(c, a.L, word_of(t)) : 0u;
#pragma unroll
            for (int q = kPlanes - 1; q >= 0; --q) {
                if (q < P) {
                    uint32_t some = 0u;
#pragma unroll
                    for (int t = 0; t < kPerLane; ++t) some |= m[t] & pl[q][t];
                    if (__any(some != 0u)) {
#pragma unroll
                        for (int t = 0; t < kPerLane; ++t) m[t] &= pl[q][t];
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < kPerLane; ++t) next[t] |= m[t];
        }
#pragma unroll
        for (int t = 0; t < kPerLane; ++t)
            if (mine(t)) acc[word_of(t)] = next[t];
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

// RULE = gbnn_rule (the counters of sum-of-sum and of the hybrid's first pass take most of the registers).
template <int RULE>
__global__ __launch_bounds__(64) void k_retrieve_generic(RetrieveArgs a)
{
    extern __shared__ uint32_t sm[];
    G g{a, (int)threadIdx.x, sm, sm + a.nw, sm + 2 * a.nw};
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
            // 32 activity bytes -> one word, in two 16-byte pieces at any alignment; the last word byte by byte
            // where the vector ends inside it
            const uint8_t *src = a.V0 + k * a.n;
            for (int w = lane; w < a.nw; w += 64) {
                uint32_t word = 0u;
                if (32 * w + 32 <= a.n) {
                    word = pack16(load16_unaligned(src + 32 * w)) | (pack16(load16_unaligned(src + 32 * w + 16)) << 16);
                } else {
                    for (int i = 32 * w; i < a.n; ++i) word |= (uint32_t)(src[i] & 1u) << (i & 31);
                }
                g.v[w] = word;
            }
        }
        __syncthreads();

        int it = 0;
        if constexpr (RULE == GBNN_SUM_OF_MAX) {
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
        } else if constexpr (RULE == GBNN_HYBRID) {
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
            // Algorithm 2, lines 1-5: the neurons of the erased clusters that receive exactly `known` signals.
            // known <= GBNN_MAX_C, so seven digits and the overflow mark decide.
            constexpr int kDigits = 7;
            static_assert(GBNN_MAX_C < (1 << kDigits), "digits of the number of known clusters");
            uint32_t pl[kDigits][kPerLane], ovf[kPerLane];
            g.template count_signals<kDigits>(pl, ovf);
#pragma unroll
            for (int t = 0; t < kPerLane; ++t) {
                if (!g.mine(t)) continue;
                const int w = g.word_of(t);
                uint32_t eq = ~ovf[t];
#pragma unroll
                for (int q = 0; q < kDigits; ++q) eq &= ((known >> q) & 1) ? pl[q][t] : ~pl[q][t];
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
                uint32_t pl[kPlanes][kPerLane], ovf[kPerLane];  // (16 digits hold any count: ovf stays 0)
                const int rows = g.template count_signals<kPlanes>(pl, ovf);
                g.sos_select(rows, pl);
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
                if (32 * w + 32 <= a.n) {
                    store16_unaligned(dst + 32 * w, spread16(word & 0xFFFFu));
                    store16_unaligned(dst + 32 * w + 16, spread16(word >> 16));
                } else {
                    for (int i = 32 * w; i < a.n; ++i) dst[i] = (uint8_t)((word >> (i & 31)) & 1u);
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
    const int64_t cap = 256 * 32;  // (one wave per workgroup: 32 fit a CU)
    if (blocks > cap) blocks = cap;
    const size_t lds = 3 * (size_t)a.nw * sizeof(uint32_t);  // three packed vectors
    if (a.rule == GBNN_SUM_OF_MAX)
        hipLaunchKernelGGL(k_retrieve_generic<GBNN_SUM_OF_MAX>, dim3((unsigned)blocks), dim3(64), lds, s, a);
    else if (a.rule == GBNN_HYBRID)
        hipLaunchKernelGGL(k_retrieve_generic<GBNN_HYBRID>, dim3((unsigned)blocks), dim3(64), lds, s, a);
    else
        hipLaunchKernelGGL(k_retrieve_generic<GBNN_SUM_OF_SUM>, dim3((unsigned)blocks), dim3(64), lds, s, a);
    return hipGetLastError();
}

}  // namespace gbnn
