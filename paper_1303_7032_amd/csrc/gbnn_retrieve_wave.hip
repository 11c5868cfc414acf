// One wavefront per probe: the whole iterate-to-fixpoint loop of a probe runs in registers.
//
// Layout.  A probe's n activity bits are held as n/32 words; lane l of the wave holds words
// l, l+64, l+128, ... ("slots" t = 0..NW-1, word index t*64 + l).  The shapes served here have
// L a power of two >= 32, so a cluster is LW = L/32 consecutive words = LW consecutive lanes of
// one slot ("group"), and 64/LW clusters share a slot.  A row of W (or of the cluster-summary
// table) in the canonical layout is then one coalesced 256-byte load per slot.
//
// All three rules are built on one primitive: walk the currently active neurons j with scalar
// code (ballot -> readlane -> count-trailing-zeros) and fetch row j of W, which by symmetry of W
// (Section IV-B) holds, for every neuron i at once, whether j signals i.
//   sum-of-max (Eq. 6-7 / bail-out-early, Section IV-D): neuron i stays on iff it is on and, for
//     every other cluster c', the OR of the rows of the active neurons of c' has bit i.  Because
//     dead neurons stay dead (Lemma 1) a cluster whose active set did not change in the previous
//     pass cannot switch anything off, so only "dirty" clusters are walked.
//   sum-of-sum (Eq. 3-5): the rows are added into bit-sliced counters (one register per binary
//     digit of the score), gamma is added to active neurons, and the per-cluster maximum is
//     found digit by digit from the top with a ballot per digit.
//   hybrid (Algorithm 2): pass 1 is the counter form restricted to "== C - e"; later passes are
//     the sum-of-max update applied to the lanes of erased clusters only.
#include "gbnn_internal.h"

namespace gbnn {
namespace {

constexpr int kPlanes = 16;  // binary digits of a score: n + gamma < 2^16 by the interface limits

__device__ __forceinline__ uint32_t readlane(uint32_t x, int l)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)x, l);
}
__device__ __forceinline__ uint64_t ballot(bool p) { return (uint64_t)__ballot(p); }

// 4 activity bytes (0/1 in bit 0) -> 4 bits, byte k -> bit k.  The multiplier places byte k's
// bit at 21+k without carries.
__device__ __forceinline__ uint32_t pack4(uint32_t x) { return (((x & 0x01010101u) * 0x00204081u) >> 21) & 0xFu; }
__device__ __forceinline__ uint32_t pack16(uint4 a)
{
    return pack4(a.x) | (pack4(a.y) << 4) | (pack4(a.z) << 8) | (pack4(a.w) << 12);
}
// 4 bits -> 4 bytes of 0/1.
__device__ __forceinline__ uint32_t spread4(uint32_t nib) { return (nib * 0x00204081u) & 0x01010101u; }
__device__ __forceinline__ uint4 spread16(uint32_t h)
{
    return make_uint4(spread4(h & 15u), spread4((h >> 4) & 15u), spread4((h >> 8) & 15u), spread4((h >> 12) & 15u));
}

template <int NW>
struct Ctx {
    const uint32_t *W;
    const uint32_t *has;
    int nw, C;
    int lane, log2lw, cps, grp, grpstart;
    uint64_t grpmask;        // low LW bits set
    bool valid[NW];          // this lane's word of slot t exists
    uint64_t validmask[NW];  // ballot of valid
    uint64_t lead[NW];       // first lane of every existing group of slot t
};

template <int NW>
__device__ __forceinline__ void load_row(const Ctx<NW> &x, const uint32_t *base, int64_t j, uint32_t (&r)[NW])
{
    const uint32_t *row = base + j * x.nw;
#pragma unroll
    for (int u = 0; u < NW; ++u) r[u] = x.valid[u] ? row[u * 64 + x.lane] : 0u;
}

// f(j) for every active neuron j held in slot t by the lanes of `lanes` (wave-uniform), ascending.
template <class F>
__device__ __forceinline__ void for_each_active(uint32_t vt, uint64_t lanes, int t, F &&f)
{
    while (lanes) {
        const int sl = __builtin_ctzll(lanes);
        lanes &= lanes - 1;
        uint32_t word = readlane(vt, sl);
        const int jb = ((t << 6) + sl) << 5;
        while (word) {
            const int b = __builtin_ctz(word);
            word &= word - 1;
            f(jb + b);
        }
    }
}

// True in every lane whose group has a set bit in the wave-uniform lane mask m.
template <int NW>
__device__ __forceinline__ bool group_any(const Ctx<NW> &x, uint64_t m)
{
    return ((m >> x.grpstart) & x.grpmask) != 0;
}

// One sum-of-max pass over the dirty clusters: acc = v AND, for each dirty cluster c',
// (OR of rows of active neurons of c'  |  own-cluster mask of c').
template <int NW>
__device__ __forceinline__ void som_pass(const Ctx<NW> &x, const uint32_t (&v)[NW], const uint64_t (&dirty)[NW],
                                         uint32_t (&acc)[NW])
{
#pragma unroll
    for (int t = 0; t < NW; ++t) acc[t] = v[t];
#pragma unroll
    for (int t = 0; t < NW; ++t) {
        const uint64_t full = ballot(v[t] == 0xFFFFFFFFu);
        const uint64_t nz = ballot(v[t] != 0u);
        uint64_t m = dirty[t];
        while (m) {
            const int g = __builtin_ctzll(m) >> x.log2lw;
            const uint64_t gl = x.grpmask << (g << x.log2lw);
            m &= ~gl;
            uint32_t R[NW];
#pragma unroll
            for (int u = 0; u < NW; ++u) R[u] = 0u;
            if ((full & gl) == gl) {
                // every neuron of the cluster is on: its contribution is the stored summary row
                load_row(x, x.has, (int64_t)(t * x.cps + g), R);
            } else {
                for_each_active(v[t], nz & gl, t, [&](int j) {
                    uint32_t r[NW];
                    load_row(x, x.W, (int64_t)j, r);
#pragma unroll
                    for (int u = 0; u < NW; ++u) R[u] |= r[u];
                });
            }
            const bool own = (x.grp == g);
#pragma unroll
            for (int u = 0; u < NW; ++u) acc[u] &= (u == t && own) ? 0xFFFFFFFFu : R[u];
        }
    }
}

// Bit-sliced sum over the rows of all active neurons: pl[p] holds digit p of
// sum_j v_j w_ji for the 32 neurons of each word.  Returns the number of active neurons.
template <int NW>
__device__ __forceinline__ int count_signals(const Ctx<NW> &x, const uint32_t (&v)[NW], uint32_t (&pl)[kPlanes][NW])
{
#pragma unroll
    for (int p = 0; p < kPlanes; ++p)
#pragma unroll
        for (int u = 0; u < NW; ++u) pl[p][u] = 0u;
    int rows = 0;
#pragma unroll
    for (int t = 0; t < NW; ++t) {
        const uint64_t nz = ballot(v[t] != 0u);
        for_each_active(v[t], nz, t, [&](int j) {
            uint32_t carry[NW];
            load_row(x, x.W, (int64_t)j, carry);
            ++rows;
            const int np = 32 - __builtin_clz((unsigned)rows);  // digits a count of `rows` can need
#pragma unroll
            for (int p = 0; p < kPlanes; ++p) {
                if (p >= np) break;
#pragma unroll
                for (int u = 0; u < NW; ++u) {
                    const uint32_t c2 = pl[p][u] & carry[u];
                    pl[p][u] ^= carry[u];
                    carry[u] = c2;
                }
            }
        });
    }
    return rows;
}

template <int NW>
__device__ __forceinline__ bool any_diff(const uint32_t (&a)[NW], const uint32_t (&b)[NW], uint64_t (&lanes)[NW])
{
    uint64_t any = 0;
#pragma unroll
    for (int t = 0; t < NW; ++t) {
        lanes[t] = ballot(a[t] != b[t]);
        any |= lanes[t];
    }
    return any != 0;
}

template <int NW, int RULE>
__global__ __launch_bounds__(256) void k_retrieve_wave(RetrieveArgs a, int log2lw)
{
    Ctx<NW> x;
    x.W = a.W;
    x.has = a.has;
    x.nw = a.nw;
    x.C = a.C;
    x.lane = threadIdx.x & 63;
    x.log2lw = log2lw;
    x.cps = 64 >> log2lw;
    x.grp = x.lane >> log2lw;
    x.grpstart = x.grp << log2lw;
    x.grpmask = (log2lw == 6) ? ~0ull : ((1ull << (1 << log2lw)) - 1ull);
#pragma unroll
    for (int t = 0; t < NW; ++t) {
        x.valid[t] = (t * 64 + x.lane) < a.nw;
        x.validmask[t] = ballot(x.valid[t]);
        x.lead[t] = ballot(x.valid[t] && (x.lane == x.grpstart));
    }
    const int64_t wave = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t nwaves = (int64_t)gridDim.x * 4;

    for (int64_t k = wave; k < a.K; k += nwaves) {
        // ---- probe load: 32 bytes per word, packed to bits
        uint32_t v[NW];
        const uint4 *src = reinterpret_cast<const uint4 *>(a.V0 + k * a.n);
#pragma unroll
        for (int t = 0; t < NW; ++t) {
            v[t] = 0u;
            if (x.valid[t]) {
                const uint4 lo = src[(t * 64 + x.lane) * 2];
                const uint4 hi = src[(t * 64 + x.lane) * 2 + 1];
                v[t] = pack16(lo) | (pack16(hi) << 16);
            }
        }

        int it = 0;
        if (RULE == GBNN_SUM_OF_MAX) {
            // Section III-C: clusters with no active neuron start fully active.
            uint64_t dirty[NW];
#pragma unroll
            for (int t = 0; t < NW; ++t) {
                const uint64_t nz = ballot(v[t] != 0u);
                if (x.valid[t] && !group_any(x, nz)) v[t] = 0xFFFFFFFFu;
                dirty[t] = x.validmask[t];
            }
            int p = 0;
            for (;;) {
                uint32_t acc[NW];
                som_pass(x, v, dirty, acc);
                ++p;
                const bool changed = any_diff(acc, v, dirty);
#pragma unroll
                for (int t = 0; t < NW; ++t) v[t] = acc[t];
                if (!changed) { it = p; break; }
                if (p == a.max_iters) { it = -p; break; }
            }
        } else if (RULE == GBNN_HYBRID) {
            // Algorithm 2.  Erased clusters = clusters with no active neuron in the probe.
            bool erased[NW];
            uint64_t erasedmask[NW];
            int known = 0;
#pragma unroll
            for (int t = 0; t < NW; ++t) {
                const uint64_t nz = ballot(v[t] != 0u);
                erased[t] = x.valid[t] && !group_any(x, nz);
                erasedmask[t] = ballot(erased[t]);
                uint64_t y = nz;
                for (int sh = 1; sh < (1 << log2lw); sh <<= 1) y |= y >> sh;  // group OR lands on its first lane
                known += __builtin_popcountll(y & x.lead[t]);
            }
            const int target = known;  // C - e
            // lines 2-5: keep the neurons of erased clusters that receive exactly C - e signals
            uint32_t pl[kPlanes][NW];
            const int rows = count_signals(x, v, pl);
            const int np = rows ? 32 - __builtin_clz((unsigned)rows) : 0;
#pragma unroll
            for (int u = 0; u < NW; ++u) {
                uint32_t eq = 0xFFFFFFFFu;
#pragma unroll
                for (int p = 0; p < kPlanes; ++p) {
                    if (p >= np) break;
                    eq &= ((target >> p) & 1) ? pl[p][u] : ~pl[p][u];
                }
                if (erased[u]) v[u] = eq;
            }
            int p = 1;
            if (p == a.max_iters) {
                it = -p;
            } else {
                // When every known cluster holds exactly one active neuron, "exactly C - e signals"
                // already means "adjacent to every known active neuron": known clusters are clean.
                uint64_t dirty[NW];
#pragma unroll
                for (int t = 0; t < NW; ++t) dirty[t] = (rows == known) ? erasedmask[t] : x.validmask[t];
                for (;;) {
                    uint32_t acc[NW];
                    som_pass(x, v, dirty, acc);
#pragma unroll
                    for (int t = 0; t < NW; ++t)
                        if (!erased[t]) acc[t] = v[t];  // known clusters are frozen
                    ++p;
                    const bool changed = any_diff(acc, v, dirty);
#pragma unroll
                    for (int t = 0; t < NW; ++t) v[t] = acc[t];
                    if (!changed) { it = p; break; }
                    if (p == a.max_iters) { it = -p; break; }
                }
            }
        } else {
            // Algorithm 1 with Eq. (3)-(5).
            int p = 0;
            for (;;) {
                uint32_t pl[kPlanes][NW];
                const int rows = count_signals(x, v, pl);
                const unsigned top = (unsigned)(rows + a.gamma);
                const int P = top ? 32 - __builtin_clz(top) : 0;
                if (a.gamma) {  // s_i += gamma * v_i : ripple add of a constant into the active neurons
#pragma unroll
                    for (int u = 0; u < NW; ++u) {
                        uint32_t cy = 0u;
#pragma unroll
                        for (int q = 0; q < kPlanes; ++q) {
                            if (q >= P) break;
                            const uint32_t g = ((a.gamma >> q) & 1) ? v[u] : 0u;
                            const uint32_t d = pl[q][u];
                            pl[q][u] = d ^ g ^ cy;
                            cy = (d & g) | (cy & (d ^ g));
                        }
                    }
                }
                // Eq. (4)-(5): per cluster keep the neurons whose score is the cluster maximum.
                uint32_t cand[NW];
#pragma unroll
                for (int u = 0; u < NW; ++u) cand[u] = x.valid[u] ? 0xFFFFFFFFu : 0u;
#pragma unroll
                for (int q = kPlanes - 1; q >= 0; --q) {
                    if (q >= P) continue;
#pragma unroll
                    for (int u = 0; u < NW; ++u) {
                        const uint32_t tt = cand[u] & pl[q][u];
                        const uint64_t nzm = ballot(tt != 0u);
                        if (group_any(x, nzm)) cand[u] = tt;
                    }
                }
                ++p;
                uint64_t diff[NW];
                const bool changed = any_diff(cand, v, diff);
#pragma unroll
                for (int t = 0; t < NW; ++t) v[t] = cand[t];
                if (!changed) { it = p; break; }
                if (p == a.max_iters) { it = -p; break; }
            }
        }

        // ---- result store
        if (a.iters && x.lane == 0) a.iters[k] = it;
        uint4 *dst = reinterpret_cast<uint4 *>(a.Vout + k * a.n);
#pragma unroll
        for (int t = 0; t < NW; ++t) {
            if (x.valid[t]) {
                dst[(t * 64 + x.lane) * 2] = spread16(v[t] & 0xFFFFu);
                dst[(t * 64 + x.lane) * 2 + 1] = spread16(v[t] >> 16);
            }
        }
    }
}

template <int NW>
hipError_t launch_nw(const RetrieveArgs &a, int log2lw, hipStream_t s)
{
    int64_t blocks = (a.K + 3) / 4;
    const int64_t cap = 256 * 8;  // 256 CUs x 8 workgroups of 4 waves = every wave slot of the chip
    if (blocks > cap) blocks = cap;
    const dim3 grid((unsigned)blocks), block(256);
    switch (a.rule) {
    case GBNN_SUM_OF_SUM:
        hipLaunchKernelGGL((k_retrieve_wave<NW, GBNN_SUM_OF_SUM>), grid, block, 0, s, a, log2lw);
        break;
    case GBNN_SUM_OF_MAX:
        hipLaunchKernelGGL((k_retrieve_wave<NW, GBNN_SUM_OF_MAX>), grid, block, 0, s, a, log2lw);
        break;
    default:
        hipLaunchKernelGGL((k_retrieve_wave<NW, GBNN_HYBRID>), grid, block, 0, s, a, log2lw);
        break;
    }
    return hipGetLastError();
}

}  // namespace

int wave_words_per_lane(int C, int L)
{
    if (L < 32 || L > 2048 || (L & (L - 1)) != 0) return 0;
    const int nw = C * (L / 32);
    if (nw <= 64) return 1;
    if (nw <= 128) return 2;
    if (nw <= 256) return 4;
    return 0;
}

hipError_t launch_retrieve_wave(const RetrieveArgs &a, int words_per_lane, hipStream_t s)
{
    if (a.K == 0) return hipSuccess;
    const int lw = a.L / 32;
    int log2lw = 0;
    while ((1 << log2lw) < lw) ++log2lw;
    switch (words_per_lane) {
    case 1: return launch_nw<1>(a, log2lw, s);
    case 2: return launch_nw<2>(a, log2lw, s);
    case 4: return launch_nw<4>(a, log2lw, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace gbnn
