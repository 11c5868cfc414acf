// Device helpers shared by the retrieval kernels: lane-mask primitives, the byte <-> bit conversion
// of activity vectors, cluster-wide OR by DPP butterflies, and bit-sliced counters.
#ifndef GBNN_DEVICE_H
#define GBNN_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gbnn {

constexpr int kPlanes = 16;   // binary digits of a score: n + gamma < 2^16 by the interface limits
constexpr int kRegPlanes = 8; // ... of which the low ones live in registers, the rest (scores >= 256) in LDS

__device__ __forceinline__ uint32_t readlane(uint32_t x, int l)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)x, l);
}
__device__ __forceinline__ uint64_t ballot(bool p) { return (uint64_t)__ballot(p); }
// Number of set bits of the wave-uniform mask m in lanes below this one.
__device__ __forceinline__ uint32_t mbcnt(uint64_t m)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

// 16 activity bytes (each 0 or 1) -> 16 bits, byte k -> bit k: byte-wise dot products with the
// weights 1,2,4,8 / 16,32,64,128 (v_dot4_u32_u8 accumulates), two bytes of result glued together.
__device__ __forceinline__ uint32_t pack16(uint4 a)
{
    uint32_t lo = __builtin_amdgcn_udot4(a.x, 0x08040201u, 0u, false);
    lo = __builtin_amdgcn_udot4(a.y, 0x80402010u, lo, false);
    uint32_t hi = __builtin_amdgcn_udot4(a.z, 0x08040201u, 0u, false);
    hi = __builtin_amdgcn_udot4(a.w, 0x80402010u, hi, false);
    return lo | (hi << 8);
}
// 4 bits -> 4 bytes of 0/1.
__device__ __forceinline__ uint32_t spread4(uint32_t nib) { return (nib * 0x00204081u) & 0x01010101u; }
__device__ __forceinline__ uint4 spread16(uint32_t h)
{
    return make_uint4(spread4(h & 15u), spread4((h >> 4) & 15u), spread4((h >> 8) & 15u), spread4((h >> 12) & 15u));
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

// Padded clusters: a register kernel holds a cluster of L neurons in Lp / 32 words, Lp = 2^k >= L.  The bits
// of word number `wi` of a cluster (its neurons 32 wi .. 32 wi + 31) that are neurons at all:
__device__ __forceinline__ uint32_t pad_mask(uint32_t L, uint32_t wi)
{
    const int left = (int)L - 32 * (int)wi;
    return left >= 32 ? 0xFFFFFFFFu : left <= 0 ? 0u : (1u << left) - 1u;
}
// 16 bytes at any alignment (the hardware takes unaligned multi-word accesses to global memory).
typedef uint32_t u32x4_unaligned __attribute__((ext_vector_type(4), aligned(1)));
__device__ __forceinline__ uint4 load16_unaligned(const uint8_t *p)
{
    const u32x4_unaligned x = *reinterpret_cast<const u32x4_unaligned *>(p);
    return make_uint4(x.x, x.y, x.z, x.w);
}
__device__ __forceinline__ void store16_unaligned(uint8_t *p, uint4 s)
{
    u32x4_unaligned x = {s.x, s.y, s.z, s.w};
    *reinterpret_cast<u32x4_unaligned *>(p) = x;
}
// 16 bytes to a 16-byte aligned address, non-temporal: not kept in the caches on the way to memory.
typedef uint32_t u32x4_aligned __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store16_nontemporal(uint8_t *p, uint4 s)
{
    const u32x4_aligned x = {s.x, s.y, s.z, s.w};
    __builtin_nontemporal_store(x, reinterpret_cast<u32x4_aligned *>(p));
}
__device__ __forceinline__ uint4 load16_nontemporal(const uint8_t *p)
{
    const u32x4_aligned x = __builtin_nontemporal_load(reinterpret_cast<const u32x4_aligned *>(p));
    return make_uint4(x.x, x.y, x.z, x.w);
}
__device__ __forceinline__ void store16_unaligned_nontemporal(uint8_t *p, uint4 s)
{
    const u32x4_unaligned x = {s.x, s.y, s.z, s.w};
    __builtin_nontemporal_store(x, reinterpret_cast<u32x4_unaligned *>(p));
}
// The first `count` (< 16) of 16 bytes, the rest zero: byte loads, none past the last one asked for.
__device__ __forceinline__ uint4 load_bytes(const uint8_t *p, uint32_t count)
{
    uint32_t d[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int b = 0; b < 15; ++b)
        if ((uint32_t)b < count) d[b >> 2] |= (uint32_t)p[b] << (8 * (b & 3));
    return make_uint4(d[0], d[1], d[2], d[3]);
}
// The 32 activity bytes cl[32 wi .. 32 wi + 31] of a cluster (cl = its first byte, any alignment) as 32
// bits; bytes past the end of the cluster (L) give 0.  A 16-byte piece that straddles the end of the cluster
// is read whole -- what follows in memory is the next cluster or the next probe -- unless `last`: the
// cluster is the last one of the last probe, and nothing past its end is touched.
__device__ __forceinline__ uint32_t load_cluster_word(const uint8_t *cl, uint32_t L, uint32_t wi, bool last)
{
    const uint32_t l0 = 32u * wi;
    uint4 p[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const uint32_t at = l0 + 16u * h;
        p[h] = make_uint4(0u, 0u, 0u, 0u);
        if (at + 16u <= L || (at < L && !last))
            p[h] = load16_unaligned(cl + at);
        else if (at < L)
            p[h] = load_bytes(cl + at, L - at);
    }
    return (pack16(p[0]) | (pack16(p[1]) << 16)) & pad_mask(L, wi);
}
// On the way from a padded kernel's words to the canonical layout (the packed output of the message boundary
// when clusters share words, the byte output of the activity boundary): word `wi` of cluster c, value v (bits
// past the end of the cluster are zero), ORed into the canonical bit positions c*L + 32 wi .. of a bit vector
// in LDS that the wave has zeroed.
__device__ __forceinline__ void or_cluster_word(uint32_t *out, uint32_t c, uint32_t L, uint32_t wi, uint32_t v)
{
    if (32u * wi >= L || v == 0u) return;
    const uint32_t pos = c * L + 32u * wi, sh = pos & 31u;
    atomicOr(out + (pos >> 5), v << sh);
    if (sh && (v >> (32u - sh))) atomicOr(out + (pos >> 5) + 1, v >> (32u - sh));
}
// LDS traffic between the lanes of one wave: make earlier writes visible to later reads.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// A wave-uniform lane mask read as a per-lane flag (no vector arithmetic: the mask is the condition).
__device__ __forceinline__ bool lane_of(uint64_t m) { return __builtin_amdgcn_inverse_ballot_w64(m); }

// OR over the 2^LG lanes of this lane's group (a group = the lanes holding one cluster), left in
// every lane of the group: a butterfly of DPP moves inside a row of 16 lanes, ds_bpermute beyond.
template <int CTRL>
__device__ __forceinline__ uint32_t or_dpp(uint32_t v)
{
    return v | (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
template <int LG>
__device__ __forceinline__ uint32_t group_or(uint32_t v)
{
    if (LG >= 1) v = or_dpp<0xB1>(v);   // quad_perm [1,0,3,2]
    if (LG >= 2) v = or_dpp<0x4E>(v);   // quad_perm [2,3,0,1]
    if (LG >= 3) v = or_dpp<0x141>(v);  // row_half_mirror
    if (LG >= 4) v = or_dpp<0x140>(v);  // row_mirror
    if (LG >= 5) v |= (uint32_t)__shfl_xor((int)v, 16);
    if (LG >= 6) v |= (uint32_t)__shfl_xor((int)v, 32);
    return v;
}

// k * m for a probe index (below 2^31 by the interface limit) and a small positive m: one 32 x 32 -> 64
// multiply instead of a 64 x 64 one.
__device__ __forceinline__ int64_t probe_offset(int64_t k, int m) { return (int64_t)((uint64_t)(uint32_t)k * (uint32_t)m); }

// Sum over the 2^LG lanes of this lane's group, left in every lane of the group (same butterfly).
template <int CTRL>
__device__ __forceinline__ uint32_t add_dpp(uint32_t v)
{
    return v + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
template <int LG>
__device__ __forceinline__ uint32_t group_add(uint32_t v)
{
    if (LG >= 1) v = add_dpp<0xB1>(v);
    if (LG >= 2) v = add_dpp<0x4E>(v);
    if (LG >= 3) v = add_dpp<0x141>(v);
    if (LG >= 4) v = add_dpp<0x140>(v);
    if (LG >= 5) v += (uint32_t)__shfl_xor((int)v, 16);
    if (LG >= 6) v += (uint32_t)__shfl_xor((int)v, 32);
    return v;
}

// The message boundary, per cluster.  word_in_cluster = index of this lane's word inside its cluster.
// Probe side: the word of a cluster whose symbol is s (anything outside [0, L) = erased, Section II-A).
__device__ __forceinline__ uint32_t symbol_word(int32_t s, uint32_t L, uint32_t word_in_cluster)
{
    const bool here = (uint32_t)s < L && ((uint32_t)s >> 5) == word_in_cluster;
    return here ? 1u << ((uint32_t)s & 31u) : 0u;
}
// Result side: the symbol of this lane's cluster given its word v of the final activity: the index of
// the active neuron if the cluster holds exactly one, -1 if none, -2 if several (Section V-B).
template <int LG>
__device__ __forceinline__ int32_t cluster_symbol(uint32_t v, uint32_t word_in_cluster)
{
    const uint32_t pc = __popc(v);
    const uint32_t tot = group_add<LG>(pc);
    const uint32_t pos = (word_in_cluster << 5) + (uint32_t)__builtin_ctz(v | 0x80000000u);
    const uint32_t possum = group_add<LG>(pc == 1u ? pos : 0u);
    return tot == 1u ? (int32_t)possum : (tot == 0u ? -1 : -2);
}

// Bit-sliced counting.  pl[q] holds binary digit q of a per-neuron counter, 32 neurons per word.
// full adder / half adder on bit vectors
// (outputs may alias inputs)
#define GBNN_FA(a, b, c, s, cy)                                        \
    {                                                                  \
        const uint32_t a_ = (a), b_ = (b), c_ = (c), t_ = a_ ^ b_;     \
        s = t_ ^ c_;                                                   \
        cy = (a_ & b_) | (c_ & t_);                                    \
    }
#define GBNN_HA(a, b, s, cy)                  \
    {                                         \
        const uint32_t a_ = (a), b_ = (b);    \
        s = a_ ^ b_;                          \
        cy = a_ & b_;                         \
    }

// Bit-sliced counters of one probe: digit q of the counter of the 32 neurons of word (slot u, this
// lane).  Digits 0..7 are registers; digits 8..15 are needed only when a score reaches 256 (hundreds
// of active neurons, or a large gamma) and live in this wave's LDS column, zero until first written.
template <int NW>
struct Planes {
    uint32_t lo[kRegPlanes][NW];
    uint32_t *hi;  // LDS, [kPlanes - kRegPlanes][NW][64], this lane's column
    int nhi;       // high digits written so far

    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int q = 0; q < kRegPlanes; ++q)
#pragma unroll
            for (int u = 0; u < NW; ++u) lo[q][u] = 0u;
        nhi = 0;
    }
    __device__ __forceinline__ uint32_t get_hi(int q, int u) const
    {
        return (q - kRegPlanes < nhi) ? hi[((q - kRegPlanes) * NW + u) * 64] : 0u;
    }
    __device__ __forceinline__ void set_hi(int q, int u, uint32_t val) { hi[((q - kRegPlanes) * NW + u) * 64] = val; }
    // digits kRegPlanes..np-1 += carry-in cy[u] (half-adder ripple); afterwards np digits are valid
    __device__ __forceinline__ void ripple_hi(uint32_t (&cy)[NW], int np)
    {
        for (int q = kRegPlanes; q < np; ++q)
#pragma unroll
            for (int u = 0; u < NW; ++u) {
                const uint32_t dgt = get_hi(q, u);
                set_hi(q, u, dgt ^ cy[u]);
                cy[u] &= dgt;
            }
        if (np - kRegPlanes > nhi) nhi = np - kRegPlanes;
    }
};

// pl += number of rows among r[0..B-1] that have the bit, for every bit position.  The B one-bit
// rows are first compressed to one small binary number with a carry-save tree, then that number is
// rippled into the counters; np = digits the counters can need afterwards.
template <int NW, int B>
__device__ __forceinline__ void add_rows(Planes<NW> &pl, const uint32_t (&r)[B][NW], int np)
{
    static_assert(B == 4 || B == 8, "batch of 4 or 8 rows");
    uint32_t cyv[NW];
#pragma unroll
    for (int u = 0; u < NW; ++u) {
        uint32_t b[4];
        int nb;
        if (B == 8) {
            uint32_t s0, c0, s1, c1, s2, c2, c3, s4, c4, c5;
            GBNN_FA(r[0][u], r[1][u], r[2][u], s0, c0);
            GBNN_FA(r[3][u], r[4][u], r[5][u], s1, c1);
            GBNN_HA(r[6][u], r[7][u], s2, c2);
            GBNN_FA(s0, s1, s2, b[0], c3);
            GBNN_FA(c0, c1, c2, s4, c4);
            GBNN_HA(c3, s4, b[1], c5);
            GBNN_HA(c4, c5, b[2], b[3]);
            nb = 4;
        } else {
            uint32_t s0, c0, c1;
            GBNN_FA(r[0][u], r[1][u], r[2][u], s0, c0);
            GBNN_HA(s0, r[3][u], b[0], c1);
            GBNN_HA(c0, c1, b[1], b[2]);
            b[3] = 0u;
            nb = 3;
        }
        uint32_t cy = 0u;
#pragma unroll
        for (int q = 0; q < kRegPlanes; ++q) {
            if (q < nb) {
                GBNN_FA(pl.lo[q][u], b[q], cy, pl.lo[q][u], cy);
            } else {
                if (q >= np) break;
                GBNN_HA(pl.lo[q][u], cy, pl.lo[q][u], cy);
            }
        }
        cyv[u] = cy;
    }
    if (np > kRegPlanes) pl.ripple_hi(cyv, np);
}

}  // namespace gbnn
#endif
