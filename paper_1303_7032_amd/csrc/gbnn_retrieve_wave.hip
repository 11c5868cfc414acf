// One wavefront per probe: the whole iterate-to-fixpoint loop of a probe runs in registers.
//
// Layout.  A probe's n activity bits are held as n/32 words; lane l of the wave holds words
// l, l+64, l+128, ... ("slots" t = 0..NW-1, word index t*64 + l).  The shapes served here have
// L a power of two >= 32, so a cluster is LW = L/32 consecutive words = LW consecutive lanes of
// one slot ("group"), and 64/LW clusters share a slot.  A row of W (or of the cluster-summary
// table) in the canonical layout is then one coalesced 256-byte load per slot.
//
// All three rules are built on one primitive: list the currently active neurons j and fetch
// row j of W, which by symmetry of W (Section IV-B) holds, for every neuron i at once, whether j
// signals i.
//   sum-of-max (Eq. 6-7 / bail-out-early, Section IV-D): neuron i stays on iff it is on and, for
//     every other cluster c', the OR of the rows of the active neurons of c' has bit i.  Because
//     dead neurons stay dead (Lemma 1) a cluster whose active set did not change in the previous
//     pass cannot switch anything off, so only "dirty" clusters are walked.
//   sum-of-sum (Eq. 3-5): the rows are added into bit-sliced counters (one register per binary
//     digit of the score), gamma is added to active neurons, and the per-cluster maximum is
//     found digit by digit from the top with a ballot per digit.
//   hybrid (Algorithm 2): pass 1 keeps the erased-cluster neurons with exactly C - e signals: the
//     AND of the known neurons' rows when each known cluster holds one active neuron, the counter
//     form otherwise; later passes are the sum-of-max update applied to erased clusters only.
//
// The kernel is bound by instruction issue, not by memory latency, so the listing of active
// neurons is done with vector code: every lane ranks its own set bits with ballot + mbcnt and
// pushes their neuron indices to lane `rank` with ds_permute; the row loop then needs one
// v_readlane and one buffer_load (row offset in the scalar-offset operand) per row.
#include <cstdlib>

#include "gbnn_internal.h"

namespace gbnn {
namespace {

constexpr int kPlanes = 16;   // binary digits of a score: n + gamma < 2^16 by the interface limits
constexpr int kInFlight = 4;  // row loads issued before the first is consumed
constexpr int kListMax = 63;  // entries of the in-register row list (lane 63 takes the idle pushes)

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
    __amdgpu_buffer_rsrc_t wrsrc;    // W as a raw buffer: loads beyond its end return 0
    __amdgpu_buffer_rsrc_t wbrsrc;   // rows 0..n-1: W with all-one intra-cluster blocks; rows n..n+C-1: the
                                     // cluster summaries (own-cluster bits included)
    int nw, C;
    uint32_t rowbytes;               // nw * 4
    uint32_t nrows;                  // n
    int lane, log2lw, log2L, cps, grp, grpstart;
    uint64_t grpmask;        // low LW bits set
    bool valid[NW];          // this lane's word of slot t exists
    uint32_t woffb[NW];      // byte offset of this lane's word of slot t in a row; 0 if it does not exist
    uint32_t myc[NW];        // cluster of this lane's word of slot t (never matched if it does not exist)
    uint64_t validmask[NW];  // ballot of valid
    uint64_t lead[NW];       // first lane of every existing group of slot t
};

// Row at byte offset `rowoff` (wave-uniform) of a table.  Lanes without a word read word 0 of the
// row: in bounds, and what they compute is never stored.
template <int NW>
__device__ __forceinline__ void load_row(const Ctx<NW> &x, __amdgpu_buffer_rsrc_t rsrc, uint32_t rowoff,
                                         uint32_t (&r)[NW])
{
#pragma unroll
    for (int u = 0; u < NW; ++u) r[u] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, x.woffb[u], rowoff, 0);
}

// True in every lane whose group has a set bit in the wave-uniform lane mask m.
template <int NW>
__device__ __forceinline__ bool group_any(const Ctx<NW> &x, uint64_t m)
{
    return ((m >> x.grpstart) & x.grpmask) != 0;
}

// Lane-mask helpers for groups (a group = the LW consecutive lanes holding one cluster).
// fold_or / fold_and leave, on the first lane of every group, the OR / AND of the group's bits.
template <int NW>
__device__ __forceinline__ uint64_t fold_or(const Ctx<NW> &x, uint64_t m)
{
    for (int sh = 1; sh < (1 << x.log2lw); sh <<= 1) m |= m >> sh;
    return m;
}
template <int NW>
__device__ __forceinline__ uint64_t fold_and(const Ctx<NW> &x, uint64_t m)
{
    for (int sh = 1; sh < (1 << x.log2lw); sh <<= 1) m &= m >> sh;
    return m;
}

// Lists the rows a pass must fetch in a register: lane i of `list` gets (row index + 1) of the
// i-th entry, lanes past the end get 0.  Entries are, slot by slot, the set bits of pw[] (row =
// neuron index, ascending) followed by one summary row (row n + c) for every lane flagged in
// sumlane[] (the first lane of a fully active cluster c).  Returns the number of entries, or -1
// if there are more than kListMax (list is then unusable).
template <int NW>
__device__ __forceinline__ int build_list(const Ctx<NW> &x, const uint32_t (&pw)[NW], const bool (&sumlane)[NW],
                                          uint32_t &list)
{
    int base = 0;
    list = 0u;
#pragma unroll
    for (int t = 0; t < NW; ++t) {
        const uint32_t pc = __popc(pw[t]);
        uint64_t mk = ballot(pc > 0u);
        if (mk) {
            // rank of this lane's first bit = bits in lower lanes = sum over k of #(lower lanes with > k bits)
            uint32_t rank = (uint32_t)base;
            int tot = 0;
            for (uint32_t k = 1; mk; ++k) {
                rank += mbcnt(mk);
                tot += __builtin_popcountll(mk);
                mk = ballot(pc > k);
            }
            base += tot;
            if (base > kListMax) return -1;
            uint32_t w = pw[t];
            do {
                const bool has = (w != 0u);
                const uint32_t j = ((uint32_t)((t << 6) + x.lane) << 5) + (uint32_t)__builtin_ctz(w | 0x80000000u);
                // forward permute: lane `rank` receives j+1; idle lanes all push 0 to lane 63
                list |= (uint32_t)__builtin_amdgcn_ds_permute((int)((has ? rank : 63u) << 2), (int)(has ? j + 1u : 0u));
                w &= w - 1u;
                ++rank;
            } while (ballot(w != 0u));
        }
        const uint64_t sm = ballot(sumlane[t]);
        if (sm) {
            const uint32_t rank = (uint32_t)base + mbcnt(sm);
            base += __builtin_popcountll(sm);
            if (base > kListMax) return -1;
            list |= (uint32_t)__builtin_amdgcn_ds_permute((int)((sumlane[t] ? rank : 63u) << 2),
                                                          (int)(sumlane[t] ? x.nrows + x.myc[t] + 1u : 0u));
        }
    }
    return base;
}

// acc &= , for every cluster c' with entries in the list, the OR of the rows of its entries.
// The rows come from the copy of W whose intra-cluster blocks are all ones, so a neuron of c'
// itself always passes.  Entries of one cluster are adjacent (the list is sorted by neuron index).
template <int NW>
__device__ __forceinline__ void apply_rows(const Ctx<NW> &x, uint32_t list, int total, uint32_t (&acc)[NW])
{
    // Lanes past the end repeat the last entry, so the loop below can always fetch kInFlight rows.
    const uint32_t jlast = readlane(list, total - 1) - 1u;
    const uint32_t jv = (x.lane < total) ? list - 1u : jlast;
    const uint32_t offv = jv * x.rowbytes;
    const uint32_t cv = (jv >= x.nrows) ? jv : (jv >> x.log2L);  // a summary row is a cluster of its own
    const uint32_t prev = (uint32_t)__shfl_up((int)cv, 1);
    const bool isfirst = (x.lane == 0) || (cv != prev);  // entry starts a new cluster
    const uint64_t first = ballot(isfirst);
    if (__builtin_popcountll(first) == total) {
        // every cluster lists one row: plain AND of the rows
        for (int i0 = 0; i0 < total; i0 += kInFlight) {
            uint32_t r[kInFlight][NW];
#pragma unroll
            for (int q = 0; q < kInFlight; ++q) load_row(x, x.wbrsrc, readlane(offv, i0 + q), r[q]);
#pragma unroll
            for (int q = 0; q < kInFlight; ++q)
#pragma unroll
                for (int u = 0; u < NW; ++u) acc[u] &= r[q][u];
        }
        return;
    }
    // General case, branch-free: R collects the OR of the current cluster's rows; at the first row
    // of the next cluster (keep == 0) it is ANDed into acc and restarted.
    const uint32_t keepv = isfirst ? 0u : 0xFFFFFFFFu;
    uint32_t R[NW];
#pragma unroll
    for (int u = 0; u < NW; ++u) R[u] = 0xFFFFFFFFu;
    for (int i0 = 0; i0 < total; i0 += kInFlight) {
        uint32_t r[kInFlight][NW];
#pragma unroll
        for (int q = 0; q < kInFlight; ++q) load_row(x, x.wbrsrc, readlane(offv, i0 + q), r[q]);
#pragma unroll
        for (int q = 0; q < kInFlight; ++q) {
            const uint32_t keep = readlane(keepv, i0 + q);
#pragma unroll
            for (int u = 0; u < NW; ++u) {
                acc[u] &= R[u] | keep;
                R[u] = (R[u] & keep) | r[q][u];
            }
        }
    }
#pragma unroll
    for (int u = 0; u < NW; ++u) acc[u] &= R[u];
}

// The same, with scalar enumeration and one row in flight: for more rows than the list holds.
template <int NW>
__device__ __forceinline__ void apply_rows_serial(const Ctx<NW> &x, const uint32_t (&pw)[NW],
                                                  const bool (&sumlane)[NW], uint32_t (&acc)[NW])
{
    uint32_t R[NW];
#pragma unroll
    for (int u = 0; u < NW; ++u) R[u] = 0xFFFFFFFFu;
    int curc = -1;
#pragma unroll
    for (int t = 0; t < NW; ++t) {
        uint64_t lanes = ballot(pw[t] != 0u);
        while (lanes) {
            const int sl = __builtin_ctzll(lanes);
            lanes &= lanes - 1;
            uint32_t word = readlane(pw[t], sl);
            const int c = (t << 6 | sl) >> x.log2lw;
            if (c != curc) {
#pragma unroll
                for (int u = 0; u < NW; ++u) {
                    acc[u] &= R[u];
                    R[u] = 0u;
                }
                curc = c;
            }
            while (word) {
                const uint32_t j = ((uint32_t)(t << 6 | sl) << 5) + (uint32_t)__builtin_ctz(word);
                word &= word - 1;
                uint32_t r[NW];
                load_row(x, x.wbrsrc, j * x.rowbytes, r);
#pragma unroll
                for (int u = 0; u < NW; ++u) R[u] |= r[u];
            }
        }
        for (uint64_t sm = ballot(sumlane[t]); sm; sm &= sm - 1) {
            const uint32_t c = (uint32_t)(t * x.cps + (__builtin_ctzll(sm) >> x.log2lw));
            uint32_t r[NW];
            load_row(x, x.wbrsrc, (x.nrows + c) * x.rowbytes, r);
#pragma unroll
            for (int u = 0; u < NW; ++u) acc[u] &= r[u];
        }
    }
#pragma unroll
    for (int u = 0; u < NW; ++u) acc[u] &= R[u];
}

// One sum-of-max pass over the dirty clusters: acc = v AND, for each dirty cluster c',
// (OR of rows of active neurons of c'  |  own-cluster mask of c').
template <int NW>
__device__ __forceinline__ void som_pass(const Ctx<NW> &x, const uint32_t (&v)[NW], const uint64_t (&dirty)[NW],
                                         uint32_t (&acc)[NW])
{
    uint32_t pw[NW];   // words that list rows to fetch: active words of dirty, not fully active clusters
    bool sumlane[NW];  // first lane of a dirty, fully active cluster: fetch its summary row instead
#pragma unroll
    for (int t = 0; t < NW; ++t) {
        acc[t] = v[t];
        pw[t] = 0u;
        sumlane[t] = false;
        if (dirty[t] == 0) continue;
        const uint64_t notfull = ballot(v[t] != 0xFFFFFFFFu);
        const uint64_t nz = ballot(v[t] != 0u);
        const bool gdirty = group_any(x, dirty[t]);
        // Fully active cluster (an erased cluster at the start of sum-of-max, Section III-C): what
        // survives it is its stored summary row.
        const bool gfull = !group_any(x, notfull);
        if (gdirty && !gfull) pw[t] = v[t];
        sumlane[t] = gdirty && gfull && x.valid[t] && (x.lane == x.grpstart);
        // A dirty cluster with no active neuron signals nobody: everything outside it goes off.
        uint64_t empty_leads = ballot(gdirty && !group_any(x, nz) && x.valid[t] && (x.lane == x.grpstart));
        for (; empty_leads; empty_leads &= empty_leads - 1) {
            const uint32_t c = (uint32_t)(t * x.cps + (__builtin_ctzll(empty_leads) >> x.log2lw));
#pragma unroll
            for (int u = 0; u < NW; ++u) acc[u] &= (x.myc[u] == c) ? 0xFFFFFFFFu : 0u;
        }
    }
    uint32_t list;
    const int total = build_list(x, pw, sumlane, list);
    if (total > 0) apply_rows(x, list, total, acc);
    else if (total < 0) apply_rows_serial(x, pw, sumlane, acc);
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
        uint64_t lanes = ballot(v[t] != 0u);
        while (lanes) {
            const int sl = __builtin_ctzll(lanes);
            lanes &= lanes - 1;
            uint32_t word = readlane(v[t], sl);
            while (word) {
                const uint32_t j = ((uint32_t)(t << 6 | sl) << 5) + (uint32_t)__builtin_ctz(word);
                word &= word - 1;
                uint32_t carry[NW];
                load_row(x, x.wrsrc, j * x.rowbytes, carry);
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
            }
        }
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
    x.nw = a.nw;
    x.C = a.C;
    x.rowbytes = (uint32_t)a.nw * 4u;
    x.wrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(a.W), 0, (int)((uint32_t)a.n * x.rowbytes),
                                                0x00020000);
    x.nrows = (uint32_t)a.n;
    x.wbrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(a.Wb), 0,
                                                 (int)((uint32_t)(a.n + a.C) * x.rowbytes), 0x00020000);
    x.lane = threadIdx.x & 63;
    x.log2lw = log2lw;
    x.log2L = log2lw + 5;
    x.cps = 64 >> log2lw;
    x.grp = x.lane >> log2lw;
    x.grpstart = x.grp << log2lw;
    x.grpmask = (log2lw == 6) ? ~0ull : ((1ull << (1 << log2lw)) - 1ull);
#pragma unroll
    for (int t = 0; t < NW; ++t) {
        x.valid[t] = (t * 64 + x.lane) < a.nw;
        x.woffb[t] = x.valid[t] ? (uint32_t)(t * 64 + x.lane) * 4u : 0u;
        x.myc[t] = x.valid[t] ? (uint32_t)(t * x.cps + x.grp) : 0xFFFFu;
        x.validmask[t] = ballot(x.valid[t]);
        x.lead[t] = ballot(x.valid[t] && (x.lane == x.grpstart));
    }
    const int64_t wave = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t nwaves = (int64_t)gridDim.x * 4;

    for (int64_t k = wave; k < a.K; k += nwaves) {
        // ---- probe load: 32 bytes per word, packed to bits
        uint32_t v[NW];
        const uint8_t *src = a.V0 + k * a.n;
#pragma unroll
        for (int t = 0; t < NW; ++t) {
            const uint4 *p = reinterpret_cast<const uint4 *>(src + x.woffb[t] * 8u);
            const uint4 lo = p[0];
            const uint4 hi = p[1];
            v[t] = x.valid[t] ? (pack16(lo) | (pack16(hi) << 16)) : 0u;
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
            uint64_t dirty[NW];
            int known = 0, nzlanes = 0;
            bool onehot = true;
#pragma unroll
            for (int t = 0; t < NW; ++t) {
                const uint64_t nz = ballot(v[t] != 0u);
                const uint64_t single = ballot(v[t] != 0u && (v[t] & (v[t] - 1u)) == 0u);
                onehot = onehot && (single == nz);
                nzlanes += __builtin_popcountll(nz);
                erased[t] = x.valid[t] && !group_any(x, nz);
                erasedmask[t] = ballot(erased[t]);
                known += __builtin_popcountll(fold_or(x, nz) & x.lead[t]);
            }
            if (onehot && nzlanes == known) {
                // Every known cluster holds exactly one active neuron (the probe contract).  Then
                // "exactly C - e signals" (lines 2-5) means "adjacent to every known active neuron":
                // the AND of their rows, which is a sum-of-max pass over the known clusters applied
                // to fully active erased clusters.
                uint32_t vi[NW], acc[NW];
#pragma unroll
                for (int t = 0; t < NW; ++t) {
                    vi[t] = erased[t] ? 0xFFFFFFFFu : v[t];
                    dirty[t] = x.validmask[t] & ~erasedmask[t];
                }
                som_pass(x, vi, dirty, acc);
#pragma unroll
                for (int t = 0; t < NW; ++t) {
                    if (erased[t]) v[t] = acc[t];
                    dirty[t] = erasedmask[t];  // known clusters have just been applied: clean
                }
            } else {
                // General probe: count the signals with bit-sliced counters, keep "== C - e".
                uint32_t pl[kPlanes][NW];
                const int rows = count_signals(x, v, pl);
                const int np = rows ? 32 - __builtin_clz((unsigned)rows) : 0;
#pragma unroll
                for (int u = 0; u < NW; ++u) {
                    uint32_t eq = 0xFFFFFFFFu;
#pragma unroll
                    for (int p = 0; p < kPlanes; ++p) {
                        if (p >= np) break;
                        eq &= ((known >> p) & 1) ? pl[p][u] : ~pl[p][u];
                    }
                    if (erased[u]) v[u] = eq;
                    dirty[u] = x.validmask[u];
                }
            }
            int p = 1;
            if (p == a.max_iters) {
                it = -p;
            } else {
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
        uint8_t *dstb = a.Vout + k * a.n;
#pragma unroll
        for (int t = 0; t < NW; ++t) {
            if (x.valid[t]) {
                uint4 *dst = reinterpret_cast<uint4 *>(dstb + x.woffb[t] * 8u);
                dst[0] = spread16(v[t] & 0xFFFFu);
                dst[1] = spread16(v[t] >> 16);
            }
        }
    }
}

template <int NW>
hipError_t launch_nw(const RetrieveArgs &a, int log2lw, hipStream_t s)
{
    int64_t blocks = (a.K + 3) / 4;
    int64_t cap = 256 * 8;  // 256 CUs x 8 workgroups of 4 waves = every wave slot of the chip
    if (const char *e = std::getenv("GBNN_GRID_BLOCKS")) {  // tuning aid
        const long v = std::atol(e);
        if (v > 0) cap = v;
    }
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
