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
//     found digit by digit from the top with a cluster-wide OR per digit.
//   hybrid (Algorithm 2): pass 1 keeps the erased-cluster neurons with exactly C - e signals: the
//     AND of the known neurons' rows when each known cluster holds one active neuron, the counter
//     form otherwise; later passes are the sum-of-max update applied to erased clusters only.
//
// The usual probe (one active neuron per known cluster, a few candidates left in the erased clusters
// by pass 1) leaves the vector form after pass 1: the later passes run on the candidates' adjacency
// matrix, one candidate per lane (candidate_passes).  Crowded clusters (dense networks) are walked
// lane by lane without a list (apply_by_cluster).
//
// The kernel is bound by instruction issue (scalar and vector instructions cost alike) on top of
// the probe and result traffic, so everything per pass is kept to a few vector instructions:
// cluster-wide flags are DPP butterflies over the lanes of a group, the listing of active neurons
// ranks set bits with ballot + mbcnt and pushes their indices to lane `rank` with ds_permute, and
// the row loop is one v_readlane plus one buffer_load (row offset in the scalar-offset operand) per row.

#include "gbnn_device.h"
#include "gbnn_internal.h"

namespace gbnn {
namespace {

constexpr int kListMax = 56;  // entries of the in-register row list (batches of 8 stay below lane 64;
                              // lane 63 takes the idle pushes)

template <int NW>
struct Ctx {
    __amdgpu_buffer_rsrc_t wbrsrc;   // the prepared table as a raw buffer.  Rows 0..n-1: W with all-one
                                     // intra-cluster blocks; rows n..n+C-1: the cluster summaries (own-cluster
                                     // bits included); row n+C: all zero
    uint32_t rowbytes;               // nw * 4
    uint32_t nrows;                  // n
    uint32_t nclusters;              // C
    int lane;
    bool valid[NW];          // this lane's word of slot t exists
    bool islead[NW];         // ... and is the first word of its cluster
    uint32_t woffb[NW];      // byte offset of this lane's word of slot t in a row; 0 if it does not exist
    uint32_t myc[NW];        // cluster of this lane's word of slot t (never matched if it does not exist)
    uint32_t bit0[NW];       // neuron index of bit 0 of this lane's word of slot t
    uint64_t validmask[NW];  // ballot of valid
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

// Does some existing group of slot t have no set bit in the lane mask m?  (The zero-field test
// (m - lo) & ~m & hi with one field per group.)
template <int NW, int LG>
__device__ __forceinline__ bool some_group_empty(const Ctx<NW> &x, int t, uint64_t m)
{
    constexpr int LW = 1 << LG;
    uint64_t lo = 0;
#pragma unroll
    for (int g = 0; g < 64; g += LW) lo |= 1ull << g;
    const uint64_t hi = lo << (LW - 1);
    m |= ~x.validmask[t];
    return ((m - lo) & ~m & hi) != 0;
}

// Takes the next chunk of rows a pass must fetch into a register list: lane i of `list` gets
// (row index + 1) of the i-th entry, lanes past the end get 0.  Entries are, slot by slot, the set
// bits of pw[] (row = neuron index, ascending) followed by one summary row (row n + c) for every
// lane flagged in summask[] (the first lane of a fully active cluster c).  At most kListMax
// entries are taken, whole words at a time and in order; what is taken is cleared from pw[] and
// summask[], so that calling again continues where this chunk stopped.  Returns the entry count; or -1,
// as soon as the set bits of pw[] are seen to number more than give_up (pw[], list are then unusable).
// first_rank, if given, receives per slot the list position of the first bit of this lane's word
// (meaningful where the word was taken).
template <int NW>
__device__ __forceinline__ int take_chunk(const Ctx<NW> &x, uint32_t (&pw)[NW], uint64_t (&summask)[NW],
                                          uint32_t &list, int give_up = 1 << 30, uint32_t *first_rank = nullptr)
{
    int base = 0;
    bool open = true;  // false once something had to be left for the next chunk
    list = 0u;
#pragma unroll
    for (int t = 0; t < NW; ++t) {
        if (!open) break;
        const uint32_t pc = __popc(pw[t]);
        uint64_t mk = ballot(pc > 0u);
        if (mk) {
            // rank of this lane's first bit = bits in lower lanes = sum over k of #(lower lanes with > k bits)
            uint32_t rank = (uint32_t)base + mbcnt(mk);
            int tot = __builtin_popcountll(mk);
            mk = ballot(pc > 1u);
            if (NW == 1 && !mk && base + tot <= kListMax) {
                // the common case, every listed word holds one bit: one round of pushes (kept to one word
                // per lane: with more slots the extra path costs registers the kernels do not have)
                if (base + tot > give_up) return -1;
                if (first_rank) first_rank[t] = rank;
                const bool has = pc > 0u;
                const uint32_t j = x.bit0[t] + (uint32_t)__builtin_ctz(pw[t] | 0x80000000u);
                list |= (uint32_t)__builtin_amdgcn_ds_permute((int)((has ? rank : 63u) << 2), (int)(has ? j + 1u : 0u));
                pw[t] = 0u;
                base += tot;
            } else {
                for (uint32_t k = 2; mk; ++k) {
                    rank += mbcnt(mk);
                    tot += __builtin_popcountll(mk);
                    mk = ballot(pc > k);
                }
                if (base + tot > give_up) return -1;
                if (first_rank) first_rank[t] = rank;
                uint32_t w = pw[t];
                if (base + tot > kListMax) {
                    // keep the words that fit entirely; the rest of this slot and all later slots wait
                    const bool fits = rank + pc <= (uint32_t)kListMax;
                    w = fits ? w : 0u;
                    tot = 0;
                    mk = ballot(w != 0u);
                    for (uint32_t k = 1; mk; ++k) {
                        tot += __builtin_popcountll(mk);
                        mk = ballot(fits && pc > k);
                    }
                    open = false;
                }
                pw[t] &= ~w;
                base += tot;
                while (ballot(w != 0u)) {
                    const bool has = (w != 0u);
                    const uint32_t j = x.bit0[t] + (uint32_t)__builtin_ctz(w | 0x80000000u);
                    // forward permute: lane `rank` receives j+1; idle lanes all push 0 to lane 63
                    list |= (uint32_t)__builtin_amdgcn_ds_permute((int)((has ? rank : 63u) << 2),
                                                                  (int)(has ? j + 1u : 0u));
                    w &= w - 1u;
                    ++rank;
                }
            }
        }
        const uint64_t sm = summask[t];
        if (open && sm) {
            const uint32_t rank = (uint32_t)base + mbcnt(sm);
            const bool mine = lane_of(sm) && rank < (uint32_t)kListMax;
            const uint64_t taken = ballot(mine);
            summask[t] = sm & ~taken;
            open = (summask[t] == 0);
            base += __builtin_popcountll(taken);
            list |= (uint32_t)__builtin_amdgcn_ds_permute((int)((mine ? rank : 63u) << 2),
                                                          (int)(mine ? x.nrows + x.myc[t] + 1u : 0u));
        }
    }
    return base;
}

// B rows (entries i0 .. i0+B-1 of the per-lane offset list; i0+B <= 64) fetched together, ANDed into acc.
template <int NW, int B>
__device__ __forceinline__ void and_batch(const Ctx<NW> &x, uint32_t offv, int i0, uint32_t (&acc)[NW])
{
    uint32_t r[B][NW];
    // a lane with nothing left on does not need its word of the rows (and then fetches nothing: half of
    // the row bytes for the hybrid rule, whose known clusters are not updated)
#pragma unroll
    for (int u = 0; u < NW; ++u) {
        if (acc[u] != 0u) {
#pragma unroll
            for (int q = 0; q < B; ++q)
                r[q][u] = __builtin_amdgcn_raw_buffer_load_b32(x.wbrsrc, x.woffb[u], readlane(offv, i0 + q), 0);
        } else {
#pragma unroll
            for (int q = 0; q < B; ++q) r[q][u] = 0u;
        }
    }
#pragma unroll
    for (int q = 0; q < B; ++q)
#pragma unroll
        for (int u = 0; u < NW; ++u) acc[u] &= r[q][u];
}
// B rows fetched together and folded into (R, acc): keep == 0 marks the first row of a cluster.
template <int NW, int B>
__device__ __forceinline__ void or_and_batch(const Ctx<NW> &x, uint32_t offv, uint32_t keepv, int i0,
                                             uint32_t (&R)[NW], uint32_t (&acc)[NW])
{
    uint32_t r[B][NW];
#pragma unroll
    for (int q = 0; q < B; ++q) load_row(x, x.wbrsrc, readlane(offv, i0 + q), r[q]);
#pragma unroll
    for (int q = 0; q < B; ++q) {
        const uint32_t keep = readlane(keepv, i0 + q);
#pragma unroll
        for (int u = 0; u < NW; ++u) {
            acc[u] &= R[u] | keep;
            R[u] = (R[u] & keep) | r[q][u];
        }
    }
}

// acc &= , for every cluster with a word in pw[] or a lane in summask[], what that cluster lets
// survive: the OR of the rows of its listed neurons, or its summary row.  The rows come from the
// copy of W whose intra-cluster blocks are all ones, so a neuron of the cluster itself always
// passes.  Rows are listed in chunks of up to kListMax and fetched 8 at a time (4 for a short
// tail): a pass is bound by its dependent memory round trips, not by a few redundant loads.
// Entries of one cluster are adjacent (ascending neuron index) but may straddle chunks: R holds
// the OR of the cluster in progress and prevc its number.  pw[] and summask[] are consumed.
template <int NW, int LG>
__device__ __forceinline__ void fetch_and_apply(const Ctx<NW> &x, uint32_t (&pw)[NW], uint64_t (&summask)[NW],
                                                uint32_t (&acc)[NW])
{
    uint32_t R[NW];
#pragma unroll
    for (int u = 0; u < NW; ++u) R[u] = 0xFFFFFFFFu;
    uint32_t prevc = 0xFFFFFFFFu;
    bool first_chunk = true;
    for (;;) {
        uint32_t list;
        const int total = take_chunk(x, pw, summask, list);
        if (total == 0) break;
        uint64_t rest = 0;
#pragma unroll
        for (int t = 0; t < NW; ++t) rest |= ballot(pw[t] != 0u) | summask[t];
        // Lanes past the end repeat the last entry, so that whole batches can always be fetched.
        const uint32_t jlast = readlane(list, total - 1) - 1u;
        const uint32_t jv = (x.lane < total) ? list - 1u : jlast;
        const uint32_t offv = __umul24(jv, x.rowbytes);
        const uint32_t cv = (jv >= x.nrows) ? jv : (jv >> (LG + 5));  // a summary row is a cluster of its own
        // cluster of the previous entry: the value of the lane below (lane 0: the last one of the previous chunk)
        const uint32_t prev = (uint32_t)__builtin_amdgcn_update_dpp((int)prevc, (int)cv, 0x138 /* wave_shr:1 */, 0xf,
                                                                    0xf, false);
        const bool isfirst = (cv != prev);  // entry starts a new cluster
        int i0 = 0;
        if (first_chunk && !rest && __builtin_popcountll(ballot(isfirst)) == total) {
            // the usual case: one chunk and every cluster lists one row: plain AND of the rows
            while (i0 < total) {
                if (total - i0 > 4) {
                    and_batch<NW, 8>(x, offv, i0, acc);
                    i0 += 8;
                } else {
                    and_batch<NW, 4>(x, offv, i0, acc);
                    i0 += 4;
                }
            }
            return;
        }
        // General case, branch-free: R collects the OR of the current cluster's rows; at the first
        // row of the next cluster (keep == 0) it is ANDed into acc and restarted.
        const uint32_t keepv = isfirst ? 0u : 0xFFFFFFFFu;
        const uint64_t starts = ballot(isfirst);  // entries that begin a cluster (lanes past the end repeat the last entry)
        while (i0 < total) {
            if (total - i0 > 4) {
                or_and_batch<NW, 8>(x, offv, keepv, i0, R, acc);
                i0 += 8;
            } else {
                or_and_batch<NW, 4>(x, offv, keepv, i0, R, acc);
                i0 += 4;
            }
            // Dense networks list tens of rows per cluster.  Once the OR of the cluster in progress covers
            // everything still on, its remaining rows cannot switch anything off: skip to the next cluster.
            if (i0 < total && !((starts >> i0) & 1ull)) {
                uint64_t uncovered = 0;
#pragma unroll
                for (int u = 0; u < NW; ++u) uncovered |= ballot((acc[u] & ~R[u]) != 0u);
                if (!uncovered) {
                    const uint64_t later = starts >> i0;
                    i0 = later ? i0 + __builtin_ctzll(later) : total;
                }
            }
        }
        if (!rest) break;
        prevc = readlane(cv, total - 1);
        first_chunk = false;
    }
#pragma unroll
    for (int u = 0; u < NW; ++u) acc[u] &= R[u];
}

// acc &= the row of the active neuron of every nonzero word of v[], for v[] whose words hold at most one
// bit each and whose clusters hold at most one active neuron each (the probe contract: one active neuron
// per known cluster), so that "for every cluster the OR of its rows" is the AND of all rows.  The rows are
// found without ranking or pushing: the nonzero lanes of a slot are a scalar mask, walked bit by bit, and
// each lane's row offset is read out of the lane.  With one word per lane the offsets go straight into the
// loads, four rows at a time (past the end the last row is repeated); with more words per lane they are
// first collected in a list, lane i holding entry i, and fetched eight (four) at a time.
template <int NW>
__device__ __forceinline__ void and_single_rows(const Ctx<NW> &x, const uint32_t (&v)[NW], uint32_t (&acc)[NW])
{
    if constexpr (NW == 1) {
        const uint32_t joff = __umul24(x.bit0[0] + (uint32_t)__builtin_ctz(v[0] | 0x80000000u), x.rowbytes);
        uint64_t m = ballot(v[0] != 0u);
        while (m) {
            uint32_t so[4];
            so[0] = readlane(joff, __builtin_ctzll(m));
            m &= m - 1ull;
#pragma unroll
            for (int q = 1; q < 4; ++q) {
                so[q] = so[q - 1];
                if (m) {
                    so[q] = readlane(joff, __builtin_ctzll(m));
                    m &= m - 1ull;
                }
            }
            if (acc[0] != 0u) {  // a lane with nothing left on does not need its word of the rows
                uint32_t r[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) r[q] = __builtin_amdgcn_raw_buffer_load_b32(x.wbrsrc, x.woffb[0], so[q], 0);
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[0] &= r[q];
            }
        }
    } else {
        uint32_t offv = 0u, last = 0u;
        int total = 0;
#pragma unroll
        for (int t = 0; t < NW; ++t) {
            const uint32_t joff = __umul24(x.bit0[t] + (uint32_t)__builtin_ctz(v[t] | 0x80000000u), x.rowbytes);
            uint64_t m = ballot(v[t] != 0u);
            while (m && total < 64) {
                last = readlane(joff, __builtin_ctzll(m));
                m &= m - 1ull;
                offv = x.lane == total ? last : offv;
                ++total;
            }
        }
        if (total == 0) return;
        offv = x.lane < total ? offv : last;  // lanes past the end repeat the last entry: whole batches can be fetched
        int i0 = 0;
        while (i0 < total) {
            if (total - i0 > 4) {
                and_batch<NW, 8>(x, offv, i0, acc);
                i0 += 8;
            } else {
                and_batch<NW, 4>(x, offv, i0, acc);
                i0 += 4;
            }
        }
    }
}

// The same update as fetch_and_apply for crowded clusters (dense networks: tens of active neurons per
// cluster, most lanes of a cluster holding some), without building a list: cluster by cluster, every
// lane of the cluster offers the row of its lowest remaining bit (a lane with none offers the all-zero
// row), the rows of all its lanes are fetched together and ORed into R, and the next round takes the
// next bits -- until R covers every neuron still on (then the rest of the cluster cannot switch
// anything off) or no bits remain.  Needs clusters of at least 4 lanes.  pw[] is consumed.
template <int NW, int LG>
__device__ __forceinline__ void apply_by_cluster(const Ctx<NW> &x, uint32_t (&pw)[NW], uint32_t (&acc)[NW])
{
    static_assert(LG >= 2, "clusters of at least 4 lanes");
    constexpr int LW = 1 << LG;        // lanes per cluster
    constexpr int B = LW < 8 ? LW : 8;  // rows fetched together
    const uint32_t zero_off = __umul24(x.nrows + x.nclusters, x.rowbytes);
#pragma unroll
    for (int t = 0; t < NW; ++t) {
        const uint32_t cluster_bits = group_or<LG>(pw[t]);  // (all lanes take part in the butterfly)
        uint64_t todo = ballot(x.islead[t] && cluster_bits != 0u);  // first lanes of the clusters to walk
        while (todo) {
            const int lead = __builtin_ctzll(todo);
            todo &= todo - 1ull;
            uint32_t R[NW];
#pragma unroll
            for (int u = 0; u < NW; ++u) R[u] = 0u;
            uint32_t w = ((x.lane ^ lead) >> LG) == 0 ? pw[t] : 0u;  // this cluster's lanes
            for (;;) {
                const uint32_t offv = w ? __umul24(x.bit0[t] + (uint32_t)__builtin_ctz(w), x.rowbytes) : zero_off;
                w &= w - 1u;  // (0 stays 0)
#pragma unroll
                for (int b0 = 0; b0 < LW; b0 += B) {
                    uint32_t r[B][NW];
#pragma unroll
                    for (int q = 0; q < B; ++q) load_row(x, x.wbrsrc, readlane(offv, lead + b0 + q), r[q]);
#pragma unroll
                    for (int q = 0; q < B; ++q)
#pragma unroll
                        for (int u = 0; u < NW; ++u) R[u] |= r[q][u];
                }
                if (!ballot(w != 0u)) break;
                uint64_t uncovered = 0;
#pragma unroll
                for (int u = 0; u < NW; ++u) uncovered |= ballot((acc[u] & ~R[u]) != 0u);
                if (!uncovered) break;
            }
#pragma unroll
            for (int u = 0; u < NW; ++u) acc[u] &= R[u];
        }
    }
}

// One sum-of-max pass from the second on.  d[] is nonzero in the lanes that changed in the previous
// pass; only the clusters holding such a lane ("dirty") can switch anything off (Lemma 1).
//   acc = v AND over dirty clusters c' of (OR of the rows of the active neurons of c' | own mask of c')
// A cluster without any active neuron signals nobody, so every neuron outside it goes off, and it
// holds none itself: acc = 0.
template <int NW, int LG>
__device__ __forceinline__ void som_step(const Ctx<NW> &x, const uint32_t (&v)[NW], const uint32_t (&d)[NW],
                                         uint32_t (&acc)[NW])
{
    bool dead = false;
#pragma unroll
    for (int t = 0; t < NW; ++t) dead = dead || some_group_empty<NW, LG>(x, t, ballot(v[t] != 0u));
    if (dead) {
#pragma unroll
        for (int t = 0; t < NW; ++t) acc[t] = 0u;
        return;
    }
    uint32_t pw[NW];
    uint64_t summask[NW];
    int holders = 0, dirty_lanes = 0;  // lanes of dirty clusters with an active neuron / all lanes of dirty clusters
#pragma unroll
    for (int t = 0; t < NW; ++t) {
        const bool dirty = group_or<LG>(d[t]) != 0u;
        acc[t] = v[t];
        pw[t] = dirty ? v[t] : 0u;
        summask[t] = 0;
        if (LG >= 2) {
            holders += __builtin_popcountll(ballot(pw[t] != 0u));
            dirty_lanes += __builtin_popcountll(ballot(dirty && x.valid[t]));
        }
    }
    if constexpr (LG >= 2) {
        // crowded clusters (3 of 4 lanes hold active neurons): walk them lane by lane instead of listing
        if (4 * holders >= 3 * dirty_lanes && holders > 8) {
            apply_by_cluster<NW, LG>(x, pw, acc);
            return;
        }
    }
    fetch_and_apply<NW, LG>(x, pw, summask, acc);
}

// d = a ^ b; returns whether they differ anywhere.
template <int NW>
__device__ __forceinline__ bool diff(const uint32_t (&a)[NW], const uint32_t (&b)[NW], uint32_t (&d)[NW])
{
    uint64_t any = 0;
#pragma unroll
    for (int t = 0; t < NW; ++t) {
        d[t] = a[t] ^ b[t];
        any |= ballot(d[t] != 0u);
    }
    return any != 0;
}

// Bit-sliced sum over the rows of all active neurons: afterwards digit q of
//   sum_j v_j w_ji  +  (number of active neurons in i's own cluster)
// for the 32 neurons i of each word: the rows are read from the table whose intra-cluster blocks
// are all ones.  The second term is the same for all neurons of a cluster, so it does not change
// which neurons reach their cluster's maximum (Eq. 4-5).  Returns the number of active neurons.
template <int NW, int LG>
__device__ __forceinline__ int count_signals(const Ctx<NW> &x, const uint32_t (&v)[NW], Planes<NW> &pl)
{
    pl.clear();
    uint32_t pw[NW];
    uint64_t summask[NW];
#pragma unroll
    for (int t = 0; t < NW; ++t) {
        pw[t] = v[t];
        summask[t] = 0;
    }
    int rows = 0;
    for (;;) {
        uint32_t list;
        const int total = take_chunk(x, pw, summask, list);
        if (total == 0) break;
        // lanes past the end point at the all-zero row of the table
        const uint32_t jv = (x.lane < total) ? list - 1u : x.nrows + x.nclusters;
        const uint32_t offv = __umul24(jv, x.rowbytes);
        int i0 = 0;
        while (i0 < total) {
            if (total - i0 > 4) {
                uint32_t r[8][NW];
#pragma unroll
                for (int q = 0; q < 8; ++q) load_row(x, x.wbrsrc, readlane(offv, i0 + q), r[q]);
                i0 += 8;
                const int upto = rows + (i0 < total ? i0 : total);
                add_rows<NW, 8>(pl, r, 32 - __builtin_clz((unsigned)upto));
            } else {
                uint32_t r[4][NW];
#pragma unroll
                for (int q = 0; q < 4; ++q) load_row(x, x.wbrsrc, readlane(offv, i0 + q), r[q]);
                i0 += 4;
                add_rows<NW, 4>(pl, r, 32 - __builtin_clz((unsigned)(rows + total)));
            }
        }
        rows += total;
    }
    return rows;
}

// eq = neurons whose count of signals (rows of the active neurons of v having their bit) is exactly
// `target` (< 128).  A 7-digit counter with a sticky overflow flag: enough to decide equality, and
// few registers.  Used by the hybrid for probes outside the one-neuron-per-known-cluster contract.
template <int NW, int LG>
__device__ __forceinline__ void signals_equal(const Ctx<NW> &x, const uint32_t (&v)[NW], int target, uint32_t (&eq)[NW])
{
    constexpr int D = 7;
    // One slot of words at a time (the rows are listed again for every slot): this path is rare, and
    // counters for all slots at once would set the register budget of the whole kernel.
#pragma unroll
    for (int u = 0; u < NW; ++u) {
        uint32_t pl[D], ovf = 0u;
#pragma unroll
        for (int q = 0; q < D; ++q) pl[q] = 0u;
        uint32_t pw[NW];
        uint64_t summask[NW];
#pragma unroll
        for (int t = 0; t < NW; ++t) {
            pw[t] = v[t];
            summask[t] = 0;
        }
        for (;;) {
            uint32_t list;
            const int total = take_chunk(x, pw, summask, list);
            if (total == 0) break;
            const uint32_t jv = (x.lane < total) ? list - 1u : x.nrows + x.nclusters;  // padding: the all-zero row
            const uint32_t offv = __umul24(jv, x.rowbytes);
            for (int i0 = 0; i0 < total; i0 += 4) {
                uint32_t r[4];
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    r[q] = __builtin_amdgcn_raw_buffer_load_b32(x.wbrsrc, x.woffb[u], readlane(offv, i0 + q), 0);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint32_t carry = r[q];
#pragma unroll
                    for (int p = 0; p < D; ++p) {
                        const uint32_t c2 = pl[p] & carry;
                        pl[p] ^= carry;
                        carry = c2;
                    }
                    ovf |= carry;
                }
            }
        }
        uint32_t e = ~ovf;
#pragma unroll
        for (int p = 0; p < D; ++p) e &= ((target >> p) & 1) ? pl[p] : ~pl[p];
        eq[u] = e;
    }
}

// Bit q of the result = bit `bitpos` of the word at byte offset `woff` of the row at byte offset
// readlane(offv, i0 + q), q < B: B single-word loads in flight together (i0 + B <= 64).  Only the lanes with
// `take` set load (the others return 0): the address unit works through a load 16 lanes at a time and skips
// idle ones.  (The row offsets are read out of the lanes before the lanes are masked.)
template <int B, int NW>
__device__ __forceinline__ uint32_t gather_bits(const Ctx<NW> &x, uint32_t woff, uint32_t offv, int i0, uint32_t bitpos,
                                                bool take)
{
    uint32_t so[B];
#pragma unroll
    for (int q = 0; q < B; ++q) so[q] = readlane(offv, i0 + q);
    uint32_t t = 0u;
    if (take) {
        uint32_t w[B];
#pragma unroll
        for (int q = 0; q < B; ++q) w[q] = __builtin_amdgcn_raw_buffer_load_b32(x.wbrsrc, woff, so[q], 0);
#pragma unroll
        for (int q = 0; q < B; ++q) t |= ((w[q] >> bitpos) & 1u) << q;
    }
    return t;
}

// The passes after the first on the adjacency matrix of the candidates (sum-of-max and hybrid).
//
// Setting: every known cluster of the probe holds one active neuron, all of them survived pass 1 (so
// they are pairwise adjacent), and pass 1 left T <= 32 active neurons ("candidates") in the erased
// clusters, at least one in each.  Every candidate is adjacent to every known neuron (pass 1 took
// the AND of their rows), and neurons that are off stay off (Lemma 1), so from here on only the
// adjacency among the candidates decides: candidate q stays on iff every other erased cluster holds
// a candidate that is still on and adjacent to q; the known neurons stay on as long as every erased
// cluster keeps a candidate (and all go off in the pass after one has lost its last: no cluster
// signals them any more).  Lane q < T holds candidate q (ascending neuron index, so a cluster is a
// run of lanes) and A = its adjacency over the candidates, bit q' = w between candidates q' and q;
// bits of its own cluster are ones (the table's intra-cluster blocks are all ones).  A pass is then
// "does A & alive have a bit in every cluster's run of positions", a zero-field test with the runs as
// fields; no further rows are fetched and no lists built.  A is filled by T gathers: for every
// candidate q' one load in which lane q reads the word of row j_q' that holds bit j_q.
// On entry p = 1 passes are done; on exit v holds the final vector and the return value is the
// iteration count to report.  `list` / T / first_rank come from take_chunk over the candidates cand[].
template <int NW, int RULE, int LG>
__device__ __forceinline__ int candidate_passes(const Ctx<NW> &x, const uint32_t (&probe)[NW],
                                                const uint32_t (&cand)[NW], const uint32_t (&first_rank)[NW],
                                                uint32_t list, int T, int max_iters, uint32_t (&v)[NW])
{
    const bool inl = x.lane < T;
    const uint32_t jlast = readlane(list, T - 1) - 1u;
    const uint32_t jq = inl ? list - 1u : jlast;  // lanes past the end repeat the last candidate
    const uint32_t cq = jq >> (LG + 5);
    const uint32_t below = (uint32_t)__builtin_amdgcn_update_dpp((int)0xFFFFFFFFu, (int)cq, 0x138 /* wave_shr:1 */, 0xf,
                                                                 0xf, false);
    const uint32_t maskT = T == 32 ? 0xFFFFFFFFu : (1u << T) - 1u;
    const uint32_t S = (uint32_t)ballot(inl && cq != below);          // first position of every cluster's run
    const uint32_t E = ((S >> 1) | (1u << (T - 1))) & maskT;          // last position of every run
    const uint32_t woff = (jq >> 5) << 2;                             // byte offset of the candidate's word in a row
    const uint32_t bitpos = jq & 31u;
    const uint32_t offv = __umul24(jq, x.rowbytes);

    // A: lane q reads, from the row of a candidate q', the one word that holds its own bit.  The loads of a
    // batch are issued before the first is waited for (a probe's time is its chain of memory round trips), and
    // only the lanes that need the word take part: the address unit works through a load 16 lanes at a time
    // and skips idle ones.
    uint32_t A;
    if (NW > 1) {
        // More words per lane: networks whose table exceeds an L2, so that every fetched word costs a line
        // over the fabric.  W is symmetric (Section IV-B): of every pair of candidates only the later one reads
        // (q' < q, from the row of the earlier one), pairs within a cluster are not read at all (ones), and the
        // other half of A is the transpose of what was read.
        const int Tr = 31 - __builtin_clz(S);   // first position of the last run: the rows of its candidates are never read
        A = 0u;
        constexpr int TB = 8;   // loads in flight together
        for (int i0 = 0; i0 < Tr; i0 += TB) {
            uint32_t so[TB], cs[TB], w[TB];
#pragma unroll
            for (int q = 0; q < TB; ++q) {
                so[q] = readlane(offv, i0 + q);
                cs[q] = readlane(cq, i0 + q);
                w[q] = 0u;
            }
#pragma unroll
            for (int q = 0; q < TB; ++q)
                if (inl && x.lane > i0 + q && cq != cs[q]) w[q] = __builtin_amdgcn_raw_buffer_load_b32(x.wbrsrc, woff, so[q], 0);
#pragma unroll
            for (int q = 0; q < TB; ++q) A |= ((w[q] >> bitpos) & 1u) << ((i0 + q) & 31);   // idle lanes: w = 0
        }
        for (int q = 1; q < T; ++q) {
            const uint32_t row_q = readlane(A, q);    // bits q' < q of candidate q
            A |= ((row_q >> (x.lane & 31)) & 1u) << q;
        }
        {   // own cluster: ones from the first to the last position of the lane's run
            const uint32_t upto = 0xFFFFFFFFu >> (31 - (x.lane & 31));                 // positions 0 .. lane
            const int st = 31 - __builtin_clz((S & upto) | 1u);
            const uint32_t after = E & ~(upto >> 1);                                    // run ends at or after lane
            const int en = after ? __builtin_ctz(after) : 31;
            A |= (0xFFFFFFFFu >> (31 - en)) & (0xFFFFFFFFu << st);
        }
    } else {
        // One word per lane (the table stays in the L2s): one batch of 8, 12, ... 32 loads, every candidate's lane
        // taking part; positions past T repeat the last candidate.
        // W is symmetric (Section IV-B): the adjacency of candidates q and q' can be read from the row of either.
        // The rows of one cluster's candidates are therefore not fetched at all -- those of the longest run D
        // = [Ds, De) of positions: every pair with one end in D is read from the row of the other end (the
        // lanes of D take part in those loads like all others), and the bits obtained there are copied to
        // the other side afterwards.  What a dense network costs here is the number of loads, not the arithmetic.
        int Ds = 0, Dn = 0;
        if (T > 16) {
            for (uint32_t rem = S; rem;) {
                const int st = __builtin_ctz(rem);
                rem &= rem - 1u;
                const int len = (rem ? __builtin_ctz(rem) : T) - st;
                if (len > Dn) {
                    Dn = len;
                    Ds = st;
                }
            }
            if (Dn < 3) Dn = 0;
        }
        const int T2 = T - Dn;  // rows to fetch: positions 0 .. Ds-1 and Ds+Dn .. T-1
        uint32_t offc = offv;
        if (Dn)  // close the gap: list position i >= Ds takes the offset of position i + Dn
            offc = x.lane < Ds ? offv : (uint32_t)__builtin_amdgcn_ds_bpermute((x.lane + Dn) << 2, (int)offv);
        uint32_t t;
        if (T2 <= 8)
            t = gather_bits<8>(x, woff, offc, 0, bitpos, inl);
        else if (T2 <= 12)
            t = gather_bits<12>(x, woff, offc, 0, bitpos, inl);
        else if (T2 <= 16)
            t = gather_bits<16>(x, woff, offc, 0, bitpos, inl);
        else if (T2 <= 20)
            t = gather_bits<20>(x, woff, offc, 0, bitpos, inl);
        else if (T2 <= 24)
            t = gather_bits<24>(x, woff, offc, 0, bitpos, inl);
        else if (T2 <= 28)
            t = gather_bits<28>(x, woff, offc, 0, bitpos, inl);
        else
            t = gather_bits<32>(x, woff, offc, 0, bitpos, inl);
        A = t;
        if (Dn) {
            const uint32_t low = (1u << Ds) - 1u, maskD = ((1u << Dn) - 1u) << Ds;
            A = (t & low) | ((t & ~low) << Dn);            // bits back at their positions, D left open
            for (int q = Ds; q < Ds + Dn; ++q) {
                const uint32_t row_q = readlane(A, q) | maskD;  // candidate q of D: adjacent to candidate q' iff bit q' (own cluster: ones)
                A |= ((row_q >> x.lane) & 1u) << q;
            }
        }
    }

    uint32_t m = maskT;          // candidates still on
    bool known_on = true;        // the known neurons (sum-of-max switches them off with an emptied cluster)
    bool changed = true;         // pass 1 counts as a change for the hybrid; for sum-of-max the caller checked
    int p = 1, it;
    for (;;) {
        if (!changed) { it = p; break; }
        if (p == max_iters) { it = -p; break; }
        ++p;
        if (((m - S) & ~m & E) != 0u) {
            // some erased cluster has no candidate left: nobody receives a signal from it
            changed = m != 0u || (RULE == GBNN_SUM_OF_MAX && known_on);
            m = 0u;
            if (RULE == GBNN_SUM_OF_MAX) known_on = false;
        } else {
            const uint32_t y = A & m;
            const uint32_t off = (uint32_t)ballot(((y - S) & ~y & E) != 0u);
            changed = (m & off) != 0u;
            m &= ~off;
        }
    }

    // final vector: the probe's known neurons (unless switched off) and the candidates still on.  The
    // candidates of a word sit at consecutive list positions from first_rank on, lowest bit first.
#pragma unroll
    for (int u = 0; u < NW; ++u) {
        uint32_t out = known_on ? probe[u] : 0u;
        uint32_t w = cand[u], pos = first_rank[u];
        while (ballot(w != 0u)) {
            const uint32_t low = w & (0u - w);
            out |= ((m >> (pos & 31u)) & 1u) ? low : 0u;
            w ^= low;
            ++pos;
        }
        v[u] = out;
    }
    return it;
}

// NW = packed words per lane, RULE = gbnn_rule, LG = log2(words per cluster).
// Register budget, waves per SIMD: sum-of-max and hybrid 8 / 8 / 5 / 2 at 1 / 2 / 4 / 8 words per lane,
// sum-of-sum 8 / 5 / 4 / 2 (at 8 its high counter digits also take all 64 KiB of a workgroup's LDS).
template <int NW, int RULE, int LG>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(NW == 1 ? 8 : NW == 2 ? (RULE == GBNN_SUM_OF_SUM ? 5 : 8) : NW == 8 ? 2 : RULE == GBNN_SUM_OF_SUM ? 4 : 5))) void
k_retrieve_wave(RetrieveArgs a)
{
    constexpr int LW = 1 << LG;
    constexpr int CPS = 64 / LW;  // clusters per slot
    // LDS, a quarter per wave: the high counter digits of sum-of-sum, one column per lane; for every rule, at
    // the end, the packed result of a network with padded clusters on its way to the canonical layout
    constexpr int kLdsWords = RULE == GBNN_SUM_OF_SUM ? 4 * (kPlanes - kRegPlanes) * NW * 64 : 4 * NW * 64;
    __shared__ uint32_t lds_words[kLdsWords];
    uint32_t *sos_hi = lds_words;
    Ctx<NW> x;
    x.rowbytes = (uint32_t)a.nwp * 4u;
    x.nrows = (uint32_t)a.np;
    x.nclusters = (uint32_t)a.C;
    x.wbrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(a.Wb), 0,
                                                 (int)((uint32_t)(a.np + a.C + kTableExtraRows) * x.rowbytes), 0x00020000);
    x.lane = threadIdx.x & 63;
    const bool padded = a.Lp != a.L;  // clusters of L neurons held in the words of Lp = 2^k > L
    const bool plain_io = !padded && a.aligned16;  // activity in aligned 16-byte pieces, none past a cluster's end
#pragma unroll
    for (int t = 0; t < NW; ++t) {
        x.valid[t] = (t * 64 + x.lane) < a.nwp;
        x.islead[t] = x.valid[t] && (x.lane & (LW - 1)) == 0;
        x.woffb[t] = x.valid[t] ? (uint32_t)(t * 64 + x.lane) * 4u : 0u;
        x.myc[t] = x.valid[t] ? (uint32_t)(t * CPS + (x.lane >> LG)) : 0xFFFFu;
        x.bit0[t] = (uint32_t)(t * 64 + x.lane) << 5;
        x.validmask[t] = ballot(x.valid[t]);
    }
    // the bits of this lane's words that are neurons (all of them unless the clusters are padded)
    uint32_t pmask[NW];
#pragma unroll
    for (int t = 0; t < NW; ++t)
        pmask[t] = !x.valid[t] ? 0u : padded ? pad_mask((uint32_t)a.L, (uint32_t)x.lane & (LW - 1)) : 0xFFFFFFFFu;
    // One probe per wave: the hardware's workgroup dispatcher balances the uneven probe times (a grid of
    // resident waves striding over the probes measured 1.1-2x slower).
    const int64_t k = (int64_t)blockIdx.x * (blockDim.x >> 6) + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    if (k >= a.K) return;
    {
        // ---- probe load: 32 bytes per word, packed to bits; or one symbol per cluster
        uint32_t v[NW];
        if (a.sym_in) {
            const int32_t *sym = a.sym_in + probe_offset(k, a.C);
#pragma unroll
            for (int t = 0; t < NW; ++t)
                v[t] = x.valid[t] ? symbol_word(sym[x.myc[t]], (uint32_t)a.L, (uint32_t)x.lane & (LW - 1)) : 0u;
        } else if (plain_io) {
            const uint8_t *src = a.V0 + probe_offset(k, a.n);
#pragma unroll
            for (int t = 0; t < NW; ++t) {
                if (a.stream_in) {
                    // two contiguous pieces of 1 KiB per slot (lane j reads 16 bytes at 16 j of each: half (j & 1)
                    // of word j / 2, and of word 32 + j / 2), non-temporal; the lanes then collect their words
                    const uint32_t first = 64u * t + ((uint32_t)x.lane >> 1);
                    const uint8_t *piece = src + 2048u * t + 16u * (uint32_t)x.lane;
                    uint4 pa = make_uint4(0u, 0u, 0u, 0u), pb = pa;
                    if (first < (uint32_t)a.nw) pa = load16_nontemporal(piece);
                    if (first + 32u < (uint32_t)a.nw) pb = load16_nontemporal(piece + 1024);
                    const uint32_t m = pack16(pa) | (pack16(pb) << 16);
                    const int s0 = (x.lane & 31) << 1;
                    const uint32_t x0 = (uint32_t)__builtin_amdgcn_ds_bpermute(s0 << 2, (int)m);
                    const uint32_t x1 = (uint32_t)__builtin_amdgcn_ds_bpermute((s0 + 1) << 2, (int)m);
                    v[t] = x.lane < 32 ? (x0 & 0xFFFFu) | (x1 << 16) : (x0 >> 16) | (x1 & 0xFFFF0000u);
                    if (!x.valid[t]) v[t] = 0u;
                } else {
                    const uint4 *p = reinterpret_cast<const uint4 *>(src + x.woffb[t] * 8u);
                    const uint4 lo = p[0];
                    const uint4 hi = p[1];
                    v[t] = x.valid[t] ? (pack16(lo) | (pack16(hi) << 16)) : 0u;
                }
            }
        } else {
            const uint8_t *src = a.V0 + probe_offset(k, a.n);
#pragma unroll
            for (int t = 0; t < NW; ++t)
                v[t] = x.valid[t] ? load_cluster_word(src + x.myc[t] * (uint32_t)a.L, (uint32_t)a.L, (uint32_t)x.lane & (LW - 1),
                                                      k == a.K - 1 && x.myc[t] == x.nclusters - 1u)
                                  : 0u;
        }

        int it = 0;
        if (RULE == GBNN_SUM_OF_MAX || RULE == GBNN_HYBRID) {
            // Erased clusters = clusters with no active neuron in the probe.
            bool erased[NW];
            uint32_t acc[NW], d[NW], probe[NW];
            // The probe contract: every known cluster holds exactly one active neuron.
            int known = 0, nzlanes = 0;
            uint64_t multi = 0;
#pragma unroll
            for (int t = 0; t < NW; ++t) {
                erased[t] = x.valid[t] && group_or<LG>(v[t]) == 0u;
                probe[t] = v[t];
                known += __builtin_popcountll(ballot(x.islead[t] && !erased[t]));
                nzlanes += __builtin_popcountll(ballot(v[t] != 0u));
                multi |= ballot((v[t] & (v[t] - 1u)) != 0u);
            }
            const bool contract = !multi && nzlanes == known;
            int p = 1;
            bool changed = true;
            if (RULE == GBNN_SUM_OF_MAX) {
                // Section III-C: erased clusters start fully active.  Pass 1: the known clusters
                // contribute the rows of their active neurons, the (fully active) erased clusters
                // their summary rows.
                uint32_t pw[NW];
                uint64_t summask[NW], anysum = 0;
                const uint64_t full = *a.full;
#pragma unroll
                for (int t = 0; t < NW; ++t) {
                    pw[t] = v[t];
                    // (a summary row that is all ones changes nothing: not fetched)
                    summask[t] = ballot(erased[t] && x.islead[t] && !((full >> (x.myc[t] & 63u)) & 1ull));
                    anysum |= summask[t];
                    if (erased[t]) v[t] = pmask[t];
                    acc[t] = v[t];
                }
                if (contract && !anysum)
                    and_single_rows<NW>(x, pw, acc);  // no summary row to fetch: the AND of the known neurons' rows
                else
                    fetch_and_apply<NW, LG>(x, pw, summask, acc);
                changed = diff(acc, v, d);
            } else {
                // Algorithm 2, lines 1-5.
                if (contract) {
                    // Every known cluster holds exactly one active neuron.  Then "exactly C - e signals"
                    // means "adjacent to every known active neuron": the AND of their rows over the erased
                    // clusters.
#pragma unroll
                    for (int t = 0; t < NW; ++t)
                        acc[t] = erased[t] ? pmask[t] : 0u;  // (known clusters are restored below: their lanes fetch nothing)
                    and_single_rows<NW>(x, v, acc);
#pragma unroll
                    for (int t = 0; t < NW; ++t) {
                        acc[t] = erased[t] ? acc[t] : v[t];
                        d[t] = erased[t] ? 1u : 0u;  // known clusters have just been applied: clean
                    }
                } else {
                    // General probe: count the signals, keep the erased-cluster neurons with exactly C - e.
                    uint32_t eq[NW];
                    signals_equal<NW, LG>(x, v, known, eq);
#pragma unroll
                    for (int u = 0; u < NW; ++u) {
                        acc[u] = erased[u] ? eq[u] : v[u];
                        d[u] = x.valid[u] ? 1u : 0u;
                    }
                }
                // the stop test is made only after a bail-out-early pass (Algorithm 2, line 13)
            }
            // The usual probe (one active neuron per known cluster, all of them still on, a few candidates
            // in every erased cluster) finishes on the candidates' adjacency matrix; any other probe, and
            // a probe whose pass 1 changed nothing, takes the general loop below.
            bool finished = false;
            if (changed && contract) {
                uint64_t lost = 0, bare = 0;
                uint32_t pw[NW];
                uint64_t summask[NW];
#pragma unroll
                for (int t = 0; t < NW; ++t) {
                    lost |= ballot(!erased[t] && acc[t] != probe[t]);
                    pw[t] = erased[t] ? acc[t] : 0u;
                    bare |= ballot(erased[t] && group_or<LG>(pw[t]) == 0u);
                    summask[t] = 0;
                }
                // a cheap lower bound of the number of candidates: lanes with one, plus lanes with two or more
                int atleast = 0;
#pragma unroll
                for (int t = 0; t < NW; ++t)
                    atleast += __builtin_popcountll(ballot(pw[t] != 0u)) +
                               __builtin_popcountll(ballot((pw[t] & (pw[t] - 1u)) != 0u));
                if (!lost && !bare && atleast <= 32) {
                    uint32_t list;
                    uint32_t cand[NW], first_rank[NW];
#pragma unroll
                    for (int t = 0; t < NW; ++t) {
                        cand[t] = pw[t];
                        first_rank[t] = 0u;
                    }
                    const int T = take_chunk(x, pw, summask, list, 32, first_rank);
                    if (T >= 1) {
                        it = candidate_passes<NW, RULE, LG>(x, probe, cand, first_rank, list, T, a.max_iters, v);
                        finished = true;
                    }
                }
            }
            while (!finished) {
#pragma unroll
                for (int t = 0; t < NW; ++t) v[t] = acc[t];
                if (!changed) { it = p; break; }
                if (p == a.max_iters) { it = -p; break; }
                som_step<NW, LG>(x, v, d, acc);
                if (RULE == GBNN_HYBRID) {
#pragma unroll
                    for (int t = 0; t < NW; ++t)
                        if (!erased[t]) acc[t] = v[t];  // known clusters are frozen
                }
                ++p;
                changed = diff(acc, v, d);
            }
        } else {
            // Algorithm 1 with Eq. (3)-(5).
            Planes<NW> pl;
            pl.hi = sos_hi + (threadIdx.x >> 6) * ((kPlanes - kRegPlanes) * NW * 64) + x.lane;
            int p = 0;
            for (;;) {
                const int rows = count_signals<NW, LG>(x, v, pl);
                const unsigned top = (unsigned)(rows + a.gamma);
                const int P = top ? 32 - __builtin_clz(top) : 0;
                if (a.gamma) {  // s_i += gamma * v_i : ripple add of a constant into the active neurons
                    uint32_t cy[NW];
#pragma unroll
                    for (int u = 0; u < NW; ++u) {
                        cy[u] = 0u;
#pragma unroll
                        for (int q = 0; q < kRegPlanes; ++q) {
                            if (q >= P) break;
                            const uint32_t g = ((a.gamma >> q) & 1) ? v[u] : 0u;
                            GBNN_FA(pl.lo[q][u], g, cy[u], pl.lo[q][u], cy[u]);
                        }
                    }
                    for (int q = kRegPlanes; q < P; ++q)
#pragma unroll
                        for (int u = 0; u < NW; ++u) {
                            const uint32_t g = ((a.gamma >> q) & 1) ? v[u] : 0u;
                            uint32_t sum;
                            GBNN_FA(pl.get_hi(q, u), g, cy[u], sum, cy[u]);
                            pl.set_hi(q, u, sum);
                        }
                    if (P - kRegPlanes > pl.nhi) pl.nhi = P - kRegPlanes;
                }
                // Eq. (4)-(5): per cluster keep the neurons whose score is the cluster maximum,
                // found digit by digit from the top.
                uint32_t cand[NW];
#pragma unroll
                for (int u = 0; u < NW; ++u) cand[u] = pmask[u];
                for (int q = P - 1; q >= kRegPlanes; --q)
#pragma unroll
                    for (int u = 0; u < NW; ++u) {
                        const uint32_t tt = cand[u] & pl.get_hi(q, u);
                        if (group_or<LG>(tt) != 0u) cand[u] = tt;
                    }
#pragma unroll
                for (int q = kRegPlanes - 1; q >= 0; --q) {
                    if (q >= P) continue;
#pragma unroll
                    for (int u = 0; u < NW; ++u) {
                        const uint32_t tt = cand[u] & pl.lo[q][u];
                        if (group_or<LG>(tt) != 0u) cand[u] = tt;
                    }
                }
                ++p;
                uint32_t d[NW];
                const bool changed = diff(cand, v, d);
#pragma unroll
                for (int t = 0; t < NW; ++t) v[t] = cand[t];
                if (!changed) { it = p; break; }
                if (p == a.max_iters) { it = -p; break; }
            }
        }

        // ---- result store
        if (a.iters && x.lane == 0) a.iters[k] = it;
        if (a.sym_in) {
            if (a.bits_out) {
                uint32_t *out = a.bits_out + probe_offset(k, a.nw);
                if (!padded) {
#pragma unroll
                    for (int t = 0; t < NW; ++t)
                        if (x.valid[t]) out[t * 64 + x.lane] = v[t];
                } else if ((a.L & 31) == 0) {
                    // whole words: the words of a cluster that exist go to their canonical places
                    const uint32_t wi = (uint32_t)x.lane & (LW - 1);
#pragma unroll
                    for (int t = 0; t < NW; ++t)
                        if (x.valid[t] && 32u * wi < (uint32_t)a.L) out[x.myc[t] * ((uint32_t)a.L >> 5) + wi] = v[t];
                } else {
                    // clusters share words: the canonical bit vector is put together in LDS
                    uint32_t *canon = lds_words + (threadIdx.x >> 6) * (kLdsWords / 4);
                    for (int w = x.lane; w < a.nw; w += 64) canon[w] = 0u;
                    wave_lds_sync();
#pragma unroll
                    for (int t = 0; t < NW; ++t)
                        if (x.valid[t]) or_cluster_word(canon, x.myc[t], (uint32_t)a.L, (uint32_t)x.lane & (LW - 1), v[t]);
                    wave_lds_sync();
                    for (int w = x.lane; w < a.nw; w += 64) out[w] = canon[w];
                }
            }
            if (a.sym_out) {
#pragma unroll
                for (int t = 0; t < NW; ++t) {
                    const int32_t sy = cluster_symbol<LG>(v[t], (uint32_t)x.lane & (LW - 1));
                    if (x.islead[t]) a.sym_out[probe_offset(k, a.C) + x.myc[t]] = sy;
                }
            }
        } else if (plain_io) {
            uint8_t *dstb = a.Vout + probe_offset(k, a.n);
            // The wave's 64 words of a slot are 2 KiB of bytes: written as two contiguous pieces of 1 KiB, lane j
            // storing 16 bytes at 16 j of each -- half (j & 1) of the word of lane j / 2 (first piece) and of lane
            // 32 + j / 2 (second piece) -- so that every store instruction covers whole lines, and as non-temporal
            // stores: the results are not read again, and left out of the caches they do not displace the table
            // and the probes (cfg3: 52 -> 41 us, cfg5: 443 -> 400 us).
#pragma unroll
            for (int t = 0; t < NW; ++t) {
                const uint32_t wa = (uint32_t)__builtin_amdgcn_ds_bpermute((x.lane >> 1) << 2, (int)v[t]);
                const uint32_t wb = (uint32_t)__builtin_amdgcn_ds_bpermute((32 + (x.lane >> 1)) << 2, (int)v[t]);
                const uint32_t sh = (x.lane & 1) * 16;
                const uint32_t first = 64u * t + ((uint32_t)x.lane >> 1);  // the word the first piece's bytes come from
                uint8_t *piece = dstb + 2048u * t + 16u * (uint32_t)x.lane;
                if (first < (uint32_t)a.nw) store16_nontemporal(piece, spread16((wa >> sh) & 0xFFFFu));
                if (first + 32u < (uint32_t)a.nw) store16_nontemporal(piece + 1024, spread16((wb >> sh) & 0xFFFFu));
            }
        } else {
            // Padded clusters, or buffers that are not 16-byte aligned: the canonical bit vector is put together in
            // LDS (as for the packed output above) and the wave writes the n bytes of the result front to back,
            // 16 neurons = 16 bytes per lane and step at whatever alignment the result has, non-temporal like the
            // aligned stores; the last n mod 16 bytes one by one.
            uint8_t *dstb = a.Vout + probe_offset(k, a.n);
            uint32_t *canon = lds_words + (threadIdx.x >> 6) * (kLdsWords / 4);
            for (int w = x.lane; w < a.nw; w += 64) canon[w] = 0u;
            wave_lds_sync();
#pragma unroll
            for (int t = 0; t < NW; ++t)
                if (x.valid[t]) or_cluster_word(canon, x.myc[t], (uint32_t)a.L, (uint32_t)x.lane & (LW - 1), v[t]);
            wave_lds_sync();
            const uint16_t *canon16 = reinterpret_cast<const uint16_t *>(canon);
            const int pieces = a.n >> 4;
            for (int j = x.lane; j < pieces; j += 64) store16_unaligned_nontemporal(dstb + 16 * j, spread16(canon16[j]));
            const int i = (pieces << 4) + x.lane;
            if (x.lane < (a.n & 15)) dstb[i] = (uint8_t)((canon[i >> 5] >> (i & 31)) & 1u);
        }
    }
}

template <int NW, int LG>
hipError_t launch_one(const RetrieveArgs &a, hipStream_t s)
{
    const int wpb = 4;  // waves per workgroup
    const int64_t blocks = (a.K + wpb - 1) / wpb;
    if (blocks > 0x7FFFFFFFll) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(64 * wpb);
    switch (a.rule) {
    case GBNN_SUM_OF_SUM:
        hipLaunchKernelGGL((k_retrieve_wave<NW, GBNN_SUM_OF_SUM, LG>), grid, block, 0, s, a);
        break;
    case GBNN_SUM_OF_MAX:
        hipLaunchKernelGGL((k_retrieve_wave<NW, GBNN_SUM_OF_MAX, LG>), grid, block, 0, s, a);
        break;
    default:
        hipLaunchKernelGGL((k_retrieve_wave<NW, GBNN_HYBRID, LG>), grid, block, 0, s, a);
        break;
    }
    return hipGetLastError();
}

// Eight words per lane (n up to 16384): clusters of 8 to 64 lanes.
template <int LG>
hipError_t launch_one8(const RetrieveArgs &a, hipStream_t s)
{
    const int wpb = 4;
    const int64_t blocks = (a.K + wpb - 1) / wpb;
    if (blocks > 0x7FFFFFFFll) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(64 * wpb);
    if (a.rule == GBNN_SUM_OF_SUM)
        hipLaunchKernelGGL((k_retrieve_wave<8, GBNN_SUM_OF_SUM, LG>), grid, block, 0, s, a);
    else if (a.rule == GBNN_SUM_OF_MAX)
        hipLaunchKernelGGL((k_retrieve_wave<8, GBNN_SUM_OF_MAX, LG>), grid, block, 0, s, a);
    else
        hipLaunchKernelGGL((k_retrieve_wave<8, GBNN_HYBRID, LG>), grid, block, 0, s, a);
    return hipGetLastError();
}
hipError_t launch_nw8(const RetrieveArgs &a, int log2lw, hipStream_t s)
{
    switch (log2lw) {
    case 3: return launch_one8<3>(a, s);
    case 4: return launch_one8<4>(a, s);
    case 5: return launch_one8<5>(a, s);
    case 6: return launch_one8<6>(a, s);
    default: return hipErrorInvalidValue;
    }
}

template <int NW>
hipError_t launch_nw(const RetrieveArgs &a, int log2lw, hipStream_t s)
{
    switch (log2lw) {
    case 0: return launch_one<NW, 0>(a, s);
    case 1: return launch_one<NW, 1>(a, s);
    case 2: return launch_one<NW, 2>(a, s);
    case 3: return launch_one<NW, 3>(a, s);
    case 4: return launch_one<NW, 4>(a, s);
    case 5: return launch_one<NW, 5>(a, s);
    case 6: return launch_one<NW, 6>(a, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

int wave_words_per_lane(int C, int L)
{
    const Geometry g = geometry(C, L);
    if (g.Lp < 32 || g.Lp > 2048 || (g.Lp & (g.Lp - 1)) != 0 || g.Lp < L) return 0;  // (not served: geometry() left L as it is)
    const int nw = g.nwp;
    if (nw <= 64) return 1;
    if (nw <= 128) return 2;
    if (nw <= 256) return 4;
    if (nw <= 512) return 8;
    return 0;
}

hipError_t launch_retrieve_wave(const RetrieveArgs &a, int words_per_lane, hipStream_t s)
{
    if (a.K == 0) return hipSuccess;
    const int lw = a.Lp / 32;
    int log2lw = 0;
    while ((1 << log2lw) < lw) ++log2lw;
    switch (words_per_lane) {
    case 1: return launch_nw<1>(a, log2lw, s);
    case 2: return launch_nw<2>(a, log2lw, s);
    case 4: return launch_nw<4>(a, log2lw, s);
    case 8: return launch_nw8(a, log2lw, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace gbnn
