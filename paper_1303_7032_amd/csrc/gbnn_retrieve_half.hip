// Half a wavefront per probe: a wave carries two probes, lanes 0-31 one and lanes 32-63 the other,
// and runs their iterate-to-fixpoint loops in lockstep, in registers.
//
// For networks of at most 1024 neurons (32 packed words) a probe fills only half of a wave.  Sharing
// the wave puts the idle lanes to work: every vector and scalar instruction (ranking set bits,
// building the row list, cluster flags, combining rows, loop control) serves two probes, and every
// memory round trip (probe load, one row fetch per batch, result store) is waited for once per pair.
// (With two words per lane the same scheme would also cover 2048 neurons; measured, the extra
// cross-lane traffic then costs more than the sharing saves, so those shapes keep one wave per probe.)
//
// Layout.  Lane g (0..31) of a half holds word g of its probe; L is a power of two >= 32, so a
// cluster is 2^LGL consecutive lanes of the half.  A row of the prepared table is one dword load
// per lane; the two halves fetch different rows with the same instruction, each lane taking the row
// offset from its half's own row list by ds_bpermute.
//
// The rules are the same as in the one-wave-per-probe kernel, built on the same primitive (list the
// active neurons j, fetch row j of the table, which by symmetry of W (Section IV-B) tells for every
// neuron i whether j signals i):
//   sum-of-max (Eq. 6-7 / bail-out-early, Section IV-D), dirty clusters only (Lemma 1);
//   sum-of-sum (Eq. 3-5) with bit-sliced counters and a digit-by-digit cluster maximum;
//   hybrid (Algorithm 2): AND of the known neurons' rows, or the counter form, then sum-of-max passes
//     with the known clusters frozen.
// Passes are numbered alike for both probes of a wave; a probe that has converged lists no rows and
// keeps its state while the other one finishes.  Per-probe scalars (row counts, flags, pass counts)
// are pairs of wave-uniform values, turned into lane masks where a lane needs "the one of my half".

#include "gbnn_device.h"
#include "gbnn_internal.h"

namespace gbnn {
namespace {

constexpr int kHalfListMax = 28;  // entries per half of the in-register row list (batches of 4 or 8 stay
                                  // within the half; its lane 31 takes the idle pushes)

__device__ __forceinline__ uint32_t lo32(uint64_t m) { return (uint32_t)m; }
__device__ __forceinline__ uint32_t hi32(uint64_t m) { return (uint32_t)(m >> 32); }
// Lane mask with the lower half set iff b0 and the upper half set iff b1.
__device__ __forceinline__ uint64_t halves(bool b0, bool b1)
{
    return (b0 ? 0x00000000FFFFFFFFull : 0ull) | (b1 ? 0xFFFFFFFF00000000ull : 0ull);
}

struct HCtx {
    __amdgpu_buffer_rsrc_t rsrc;  // the prepared table as a raw buffer (rows 0..n-1: W with all-one
                                  // intra-cluster blocks; n..n+C-1: cluster summaries; n+C: zeros; n+C+1: ones)
    uint32_t rowbytes;            // nw * 4
    uint32_t nrows;               // n
    uint32_t zero_row, ones_row;  // row numbers of the all-zero and the all-one row
    uint32_t gl;                  // lane within the half
    uint32_t upperm;              // all ones in the lanes of the upper half
    uint32_t basev;               // ds_bpermute byte address of lane 0 of this lane's half
    bool valid;                   // this lane holds a word of an existing probe
    bool islead;                  // ... and is the first lane of its cluster
    uint32_t woffb;               // byte offset of this lane's word in a row; 0 if it holds none
    uint32_t myc;                 // cluster of this lane
    uint32_t bit0;                // neuron index of bit 0 of this lane's word

    // s0 in the lanes of the lower half, s1 in those of the upper half
    __device__ __forceinline__ uint32_t mine(uint32_t s0, uint32_t s1) const { return (s1 & upperm) | (s0 & ~upperm); }
};

// This lane's word of the row at byte offset `off` of the table.  Lanes without a word read word 0 of
// the row: in bounds, and what they compute is never stored.
__device__ __forceinline__ uint32_t load_row_h(const HCtx &x, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b32(x.rsrc, off + x.woffb, 0, 0);
}

// The value that lane addr/4 holds of a per-lane list (addr = basev + 4*i: entry i of this lane's half).
__device__ __forceinline__ uint32_t entry(uint32_t listv, uint32_t addr)
{
    return (uint32_t)__builtin_amdgcn_ds_bpermute((int)addr, (int)listv);
}

// Takes the next chunk of rows each half must fetch into a register list: lane i of a half gets
// (row number + 1) of that half's i-th entry, lanes past the end get 0.  Entries of a half are the set
// bits of its lanes' pw (row = neuron index, ascending) followed by one summary row (row n + c) for
// every lane flagged in summask (the first lane of a fully active cluster c).  At most kHalfListMax
// entries per half are taken, in order; what is taken is cleared from pw and summask, so that
// calling again continues where this chunk stopped.  tot0 / tot1 = entries taken.  first_rank, if
// given, receives the list position (within the half) of the first bit of this lane's word.
__device__ __forceinline__ void take_chunk_h(const HCtx &x, uint32_t &pw, uint64_t &summask, uint32_t &list,
                                             uint32_t &tot0, uint32_t &tot1, uint32_t *first_rank = nullptr)
{
    constexpr uint32_t kMax = (uint32_t)kHalfListMax;
    list = 0u;
    uint32_t t0 = 0, t1 = 0;
    const uint32_t pc = __popc(pw);
    uint64_t mk = ballot(pc > 0u);
    if (mk) {
        // rank of this lane's first bit = bits in lower lanes of the half
        //   = sum over k of #(lower lanes with > k bits), minus what the other half contributed
        uint32_t rank = 0;
        for (uint32_t k = 1; mk; ++k) {
            rank += mbcnt(mk);
            t0 += __popc(lo32(mk));
            t1 += __popc(hi32(mk));
            mk = ballot(pc > k);
        }
        rank -= t0 & x.upperm;
        if (first_rank) *first_rank = rank;
        // every lane pushes its bits, lowest first, while their ranks are below the limit
        uint32_t w = pw;
        for (;;) {
            const bool has = (w != 0u) && rank < kMax;
            if (!ballot(has)) break;
            const uint32_t j = x.bit0 + (uint32_t)__builtin_ctz(w | 0x80000000u);
            // forward permute: lane `rank` of the half receives j+1; idle lanes push 0 to lane 31 of the half
            list |= (uint32_t)__builtin_amdgcn_ds_permute((int)(x.basev + ((has ? rank : 31u) << 2)),
                                                          (int)(has ? j + 1u : 0u));
            w = has ? (w & (w - 1u)) : w;
            ++rank;
        }
        pw = w;
        t0 = t0 < kMax ? t0 : kMax;
        t1 = t1 < kMax ? t1 : kMax;
    }
    if (summask) {
        const uint64_t sm = summask;
        const uint32_t rank = x.mine(t0, t1) + mbcnt(sm) - ((uint32_t)__popc(lo32(sm)) & x.upperm);
        const bool take = lane_of(sm) && rank < kMax;
        const uint64_t taken = ballot(take);
        summask = sm & ~taken;
        t0 += __popc(lo32(taken));
        t1 += __popc(hi32(taken));
        list |= (uint32_t)__builtin_amdgcn_ds_permute((int)(x.basev + ((take ? rank : 31u) << 2)),
                                                      (int)(take ? x.nrows + x.myc + 1u : 0u));
    }
    tot0 = t0;
    tot1 = t1;
}

// B rows per half (entries i0 .. i0+B-1 of each half's offset list; i0+B <= 32) fetched together and
// ANDed into acc.  addr0 = bpermute address of entry i0 of this lane's half.
template <int B>
__device__ __forceinline__ void and_batch_h(const HCtx &x, uint32_t offv, uint32_t addr0, uint32_t &acc)
{
    uint32_t e[B], r[B];
#pragma unroll
    for (int q = 0; q < B; ++q) e[q] = entry(offv, addr0 + 4u * q);
#pragma unroll
    for (int q = 0; q < B; ++q) r[q] = load_row_h(x, e[q]);
#pragma unroll
    for (int q = 0; q < B; ++q) acc &= r[q];
}
// B rows per half fetched together and folded into (R, acc): keep == 0 marks the first row of a cluster.
template <int B>
__device__ __forceinline__ void or_and_batch_h(const HCtx &x, uint32_t offv, uint32_t keepv, uint32_t addr0, uint32_t &R,
                                               uint32_t &acc)
{
    uint32_t e[B], kp[B], r[B];
#pragma unroll
    for (int q = 0; q < B; ++q) e[q] = entry(offv, addr0 + 4u * q);
#pragma unroll
    for (int q = 0; q < B; ++q) kp[q] = entry(keepv, addr0 + 4u * q);
#pragma unroll
    for (int q = 0; q < B; ++q) r[q] = load_row_h(x, e[q]);
#pragma unroll
    for (int q = 0; q < B; ++q) {
        acc &= R | kp[q];
        R = (R & kp[q]) | r[q];
    }
}

// acc &= , for every cluster with a bit in pw or a lane in summask, what that cluster lets survive: the
// OR of the rows of its listed neurons, or its summary row (rows of the table whose intra-cluster
// blocks are all ones, so a neuron of the cluster itself always passes).  Both halves at once, each
// with its own list.  Entries of one cluster are adjacent (ascending neuron index) but may straddle
// chunks: R holds the OR of the cluster in progress and prevc its number.  A half with fewer entries
// than the other repeats its last one (OR and AND do not mind); a half with none reads the all-one row
// as a cluster of its own, which also closes the cluster it had in progress.  pw, summask consumed.
template <int LGL>
__device__ __forceinline__ void fetch_and_apply_h(const HCtx &x, uint32_t &pw, uint64_t &summask, uint32_t &acc)
{
    uint32_t R = 0xFFFFFFFFu;
    uint32_t prevc = 0xFFFFFFFFu;
    bool first_chunk = true;
    for (;;) {
        uint32_t list, tot0, tot1;
        take_chunk_h(x, pw, summask, list, tot0, tot1);
        if ((tot0 | tot1) == 0u) break;
        const uint64_t rest = ballot(pw != 0u) | summask;
        const uint32_t totv = x.mine(tot0, tot1);
        const bool inlist = x.gl < totv;
        const uint32_t lastaddr = x.basev + ((totv - 1u) << 2);
        const uint32_t last = entry(list, lastaddr);  // (garbage when totv == 0: not used then)
        const uint32_t jv = (inlist ? list : (totv ? last : x.ones_row + 1u)) - 1u;
        const uint32_t offv = __umul24(jv, x.rowbytes);
        const uint32_t cv = (jv >= x.nrows) ? jv : (jv >> (LGL + 5));  // a summary / padding row is a cluster of its own
        // cluster of the previous entry: the value of the lane below (lane 0 of a half: the last one of the previous chunk)
        const uint32_t below = (uint32_t)__builtin_amdgcn_update_dpp((int)prevc, (int)cv, 0x138 /* wave_shr:1 */, 0xf,
                                                                     0xf, false);
        const uint32_t prev = (x.gl == 0u) ? prevc : below;
        const bool isfirst = (cv != prev);  // entry starts a new cluster
        const uint32_t tmax = tot0 > tot1 ? tot0 : tot1;
        uint32_t addr = x.basev;
        if (first_chunk && !rest && ballot(inlist && !isfirst) == 0ull) {
            // the usual case: one chunk and every cluster lists one row: plain AND of the rows
            for (uint32_t i0 = 0; i0 < tmax;) {
                if (tmax - i0 > 4u) {
                    and_batch_h<8>(x, offv, addr, acc);
                    i0 += 8u;
                    addr += 32u;
                } else {
                    and_batch_h<4>(x, offv, addr, acc);
                    i0 += 4u;
                    addr += 16u;
                }
            }
            return;
        }
        // General case, branch-free: R collects the OR of the current cluster's rows; at the first
        // row of the next cluster (keep == 0) it is ANDed into acc and restarted.
        const uint32_t keepv = isfirst ? 0u : 0xFFFFFFFFu;
        for (uint32_t i0 = 0; i0 < tmax;) {
            if (tmax - i0 > 4u) {
                or_and_batch_h<8>(x, offv, keepv, addr, R, acc);
                i0 += 8u;
                addr += 32u;
            } else {
                or_and_batch_h<4>(x, offv, keepv, addr, R, acc);
                i0 += 4u;
                addr += 16u;
            }
        }
        if (!rest) break;
        const uint32_t lastc = entry(cv, lastaddr);
        prevc = totv ? lastc : prevc;
        first_chunk = false;
    }
    acc &= R;
}

// One sum-of-max pass from the second on, for both halves.  d is nonzero in the lanes that changed in
// the previous pass; only the clusters holding such a lane ("dirty") can switch anything off (Lemma 1).
//   acc = v AND over dirty clusters c' of (OR of the rows of the active neurons of c' | own mask of c')
// A cluster without any active neuron signals nobody, so every neuron outside it goes off, and it
// holds none itself: acc = 0 for that probe.
template <int LGL>
__device__ __forceinline__ uint32_t som_step_h(const HCtx &x, uint32_t v, uint32_t d)
{
    const uint64_t em = ballot(x.valid && group_or<LGL>(v) == 0u);
    const bool deadlane = lane_of(halves(lo32(em) != 0u, hi32(em) != 0u));
    const bool dirty = group_or<LGL>(d) != 0u;
    uint32_t acc = v;
    uint32_t pw = (dirty && !deadlane) ? v : 0u;
    uint64_t summask = 0;
    fetch_and_apply_h<LGL>(x, pw, summask, acc);
    return deadlane ? 0u : acc;
}

// Bit-sliced sum over the rows of all active neurons of v (both halves, each its own rows): afterwards
// digit q of   sum_j v_j w_ji  +  (number of active neurons in i's own cluster)   for the 32 neurons i
// of this lane's word: the rows are read from the table whose intra-cluster blocks are all ones.  The
// second term is the same for all neurons of a cluster, so it does not change which neurons reach
// their cluster's maximum (Eq. 4-5).  A half with fewer rows reads the all-zero row.  Returns the
// larger of the two halves' numbers of active neurons.
__device__ __forceinline__ uint32_t count_signals_h(const HCtx &x, uint32_t v, Planes<1> &pl)
{
    pl.clear();
    uint32_t pw = v;
    uint64_t summask = 0;
    uint32_t rows0 = 0, rows1 = 0;
    for (;;) {
        uint32_t list, tot0, tot1;
        take_chunk_h(x, pw, summask, list, tot0, tot1);
        if ((tot0 | tot1) == 0u) break;
        const uint32_t totv = x.mine(tot0, tot1);
        const uint32_t jv = (x.gl < totv) ? list - 1u : x.zero_row;
        const uint32_t offv = __umul24(jv, x.rowbytes);
        const uint32_t tmax = tot0 > tot1 ? tot0 : tot1;
        const uint32_t before = rows0 > rows1 ? rows0 : rows1;
        uint32_t addr = x.basev;
        for (uint32_t i0 = 0; i0 < tmax;) {
            if (tmax - i0 > 4u) {
                uint32_t e[8], r[8][1];
#pragma unroll
                for (int q = 0; q < 8; ++q) e[q] = entry(offv, addr + 4u * q);
#pragma unroll
                for (int q = 0; q < 8; ++q) r[q][0] = load_row_h(x, e[q]);
                i0 += 8u;
                addr += 32u;
                const uint32_t upto = before + (i0 < tmax ? i0 : tmax);
                add_rows<1, 8>(pl, r, 32 - __builtin_clz(upto));
            } else {
                uint32_t e[4], r[4][1];
#pragma unroll
                for (int q = 0; q < 4; ++q) e[q] = entry(offv, addr + 4u * q);
#pragma unroll
                for (int q = 0; q < 4; ++q) r[q][0] = load_row_h(x, e[q]);
                i0 += 4u;
                addr += 16u;
                add_rows<1, 4>(pl, r, 32 - __builtin_clz(before + tmax));
            }
        }
        rows0 += tot0;
        rows1 += tot1;
    }
    return rows0 > rows1 ? rows0 : rows1;
}

// The neurons whose count of signals (rows of the active neurons of v having their bit) is exactly
// this lane's `target` (< 128).  A 7-digit counter with a sticky overflow flag: enough to decide
// equality, and few registers.  Used by the hybrid for probes outside the one-neuron-per-known-cluster
// contract.
__device__ __forceinline__ uint32_t signals_equal_h(const HCtx &x, uint32_t v, uint32_t target)
{
    constexpr int D = 7;
    uint32_t pl[D], ovf = 0u;
#pragma unroll
    for (int q = 0; q < D; ++q) pl[q] = 0u;
    uint32_t pw = v;
    uint64_t summask = 0;
    for (;;) {
        uint32_t list, tot0, tot1;
        take_chunk_h(x, pw, summask, list, tot0, tot1);
        if ((tot0 | tot1) == 0u) break;
        const uint32_t totv = x.mine(tot0, tot1);
        const uint32_t jv = (x.gl < totv) ? list - 1u : x.zero_row;  // padding: the all-zero row
        const uint32_t offv = __umul24(jv, x.rowbytes);
        const uint32_t tmax = tot0 > tot1 ? tot0 : tot1;
        uint32_t addr = x.basev;
        for (uint32_t i0 = 0; i0 < tmax; i0 += 4u, addr += 16u) {
            uint32_t e[4], r[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) e[q] = entry(offv, addr + 4u * q);
#pragma unroll
            for (int q = 0; q < 4; ++q) r[q] = load_row_h(x, e[q]);
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
    uint32_t eq = ~ovf;
#pragma unroll
    for (int p = 0; p < D; ++p) {
        const uint32_t want = 0u - ((target >> p) & 1u);  // all ones iff digit p of the target is 1
        eq &= ~(pl[p] ^ want);
    }
    return eq;
}

// The passes after the first on the adjacency matrices of the candidates, for both probes of the wave
// (the method of the one-wave-per-probe kernel: there a probe qualifies when every known cluster holds
// one active neuron, all still on after pass 1, and pass 1 left a few candidates in every erased
// cluster).  Lane q of a half holds candidate q of its probe and A, its adjacency over that probe's
// candidates, filled by gathers: for candidate q' one load in which lane q reads the word of row j_q'
// that holds bit j_q, the row offset coming from the half's list.  A pass is the zero-field test of
// A & alive over the clusters' runs of list positions.  live0 / live1: the probe still runs after
// pass 1 (else it is finished: it keeps `fin` and reports 1 pass).  On exit v is the final vector.
template <int RULE, int LGL>
__device__ __forceinline__ void candidate_passes_h(const HCtx &x, uint32_t probe, uint32_t cand, uint32_t first_rank,
                                                   uint32_t list, uint32_t T0, uint32_t T1, bool live0, bool live1,
                                                   uint32_t fin, int max_iters, uint32_t &v, int &it0, int &it1)
{
    const uint32_t Tv = x.mine(T0, T1);
    const bool inl = x.gl < Tv;
    const uint32_t last = entry(list, x.basev + ((Tv - 1u) << 2));      // (garbage when Tv == 0: not used then)
    const uint32_t jq = (inl ? list : (Tv ? last : 1u)) - 1u;            // lanes past the end repeat the last candidate
    const uint32_t cq = jq >> (LGL + 5);
    const uint32_t below = (uint32_t)__builtin_amdgcn_update_dpp((int)0xFFFFFFFFu, (int)cq, 0x138 /* wave_shr:1 */, 0xf,
                                                                 0xf, false);
    const uint64_t startm = ballot(inl && (x.gl == 0u || cq != below));  // first position of every cluster's run
    const uint32_t S0 = lo32(startm), S1 = hi32(startm);
    const uint32_t full0 = (1u << T0) - 1u, full1 = (1u << T1) - 1u;     // T <= kHalfListMax < 32
    const uint32_t E0 = T0 ? ((S0 >> 1) | (1u << (T0 - 1u))) & full0 : 0u;  // last position of every run
    const uint32_t E1 = T1 ? ((S1 >> 1) | (1u << (T1 - 1u))) & full1 : 0u;
    const uint32_t woff = (jq >> 5) << 2;
    const uint32_t bitpos = jq & 31u;
    const uint32_t offv = __umul24(jq, x.rowbytes);
    const uint32_t Tmax = T0 > T1 ? T0 : T1;

    uint32_t A = 0u;
    uint32_t addr = x.basev;
    for (uint32_t i0 = 0; i0 < Tmax; i0 += 4u, addr += 16u) {
        uint32_t e[4], w[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) e[q] = entry(offv, addr + 4u * q);
#pragma unroll
        for (int q = 0; q < 4; ++q) w[q] = __builtin_amdgcn_raw_buffer_load_b32(x.rsrc, e[q] + woff, 0, 0);
        uint32_t t = 0u;
#pragma unroll
        for (int q = 0; q < 4; ++q) t |= ((w[q] >> bitpos) & 1u) << q;
        A |= t << i0;
    }

    uint32_t m0 = live0 ? full0 : 0u, m1 = live1 ? full1 : 0u;  // candidates still on
    bool kon0 = true, kon1 = true;                              // the known neurons (sum-of-max can switch them off)
    bool chg0 = live0, chg1 = live1;
    bool done0 = false, done1 = false;
    const uint32_t Sv = x.mine(S0, S1), Ev = x.mine(E0, E1);
    for (int p = 1;;) {
        if (!done0 && (!chg0 || p == max_iters)) {
            it0 = chg0 ? -p : p;
            done0 = true;
        }
        if (!done1 && (!chg1 || p == max_iters)) {
            it1 = chg1 ? -p : p;
            done1 = true;
        }
        if (done0 && done1) break;
        ++p;
        const uint32_t y = A & x.mine(m0, m1);
        const uint64_t offm = ballot(((y - Sv) & ~y & Ev) != 0u);
        if (!done0) {
            if (((m0 - S0) & ~m0 & E0) != 0u) {  // an erased cluster has no candidate left: nobody hears from it
                chg0 = m0 != 0u || (RULE == GBNN_SUM_OF_MAX && kon0);
                m0 = 0u;
                if (RULE == GBNN_SUM_OF_MAX) kon0 = false;
            } else {
                chg0 = (m0 & lo32(offm)) != 0u;
                m0 &= ~lo32(offm);
            }
        }
        if (!done1) {
            if (((m1 - S1) & ~m1 & E1) != 0u) {
                chg1 = m1 != 0u || (RULE == GBNN_SUM_OF_MAX && kon1);
                m1 = 0u;
                if (RULE == GBNN_SUM_OF_MAX) kon1 = false;
            } else {
                chg1 = (m1 & hi32(offm)) != 0u;
                m1 &= ~hi32(offm);
            }
        }
    }

    // final vector: the probe's known neurons (unless switched off) and the candidates still on; the
    // candidates of a word sit at consecutive list positions from first_rank on, lowest bit first
    uint32_t out = lane_of(halves(kon0, kon1)) ? probe : 0u;
    const uint32_t mv = x.mine(m0, m1);
    uint32_t w = cand, pos = first_rank;
    while (ballot(w != 0u)) {
        const uint32_t low = w & (0u - w);
        out |= ((mv >> (pos & 31u)) & 1u) ? low : 0u;
        w ^= low;
        ++pos;
    }
    v = lane_of(halves(live0, live1)) ? out : fin;
}

// RULE = gbnn_rule, LGL = log2(lanes per cluster) = log2(L / 32).
template <int RULE, int LGL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(8))) void k_retrieve_half(RetrieveArgs a)
{
    // LDS, a quarter per wave: the high counter digits of sum-of-sum, one column per lane; for every rule, at
    // the end, the packed results of a network with padded clusters on their way to the canonical layout
    constexpr int kLdsWords = RULE == GBNN_SUM_OF_SUM ? 4 * (kPlanes - kRegPlanes) * 64 : 4 * 64;
    __shared__ uint32_t lds_words[kLdsWords];
    uint32_t *sos_hi = lds_words;
    const int wpb = (int)(blockDim.x >> 6);  // waves per workgroup
    const int64_t pair = (int64_t)blockIdx.x * wpb + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t k0 = pair * 2;  // probes k0 (lower half) and k0 + 1 (upper half)
    if (k0 >= a.K) return;

    HCtx x;
    const uint32_t lane = threadIdx.x & 63u;
    const bool upper = lane >= 32u;
    x.gl = lane & 31u;
    x.upperm = upper ? 0xFFFFFFFFu : 0u;
    x.basev = upper ? 128u : 0u;
    x.rowbytes = (uint32_t)a.nwp * 4u;
    x.nrows = (uint32_t)a.np;
    x.zero_row = (uint32_t)(a.np + a.C);
    x.ones_row = x.zero_row + 1u;
    x.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(a.Wb), 0,
                                               (int)((uint32_t)(a.np + a.C + kTableExtraRows) * x.rowbytes), 0x00020000);
    const bool pvalid = k0 + (upper ? 1 : 0) < a.K;  // K odd: the last wave carries one probe
    x.valid = pvalid && x.gl < (uint32_t)a.nwp;
    x.islead = x.valid && (x.gl & ((1u << LGL) - 1u)) == 0u;
    x.woffb = x.valid ? x.gl * 4u : 0u;
    x.myc = x.gl >> LGL;
    x.bit0 = x.gl * 32u;

    // ---- probe load: 32 bytes per lane, packed to bits; or one symbol per cluster
    const int second = (pvalid && upper) ? 1 : 0;  // this lane's probe is k0 + second
    const int64_t kmine = k0 + second;
    const uint32_t boff = (upper ? (uint32_t)a.n : 0u) + x.woffb * 8u;  // this lane's bytes, from the first probe of the pair
    constexpr uint32_t kInCluster = (1u << LGL) - 1u;
    const bool padded = a.Lp != a.L;  // clusters of L neurons held in the words of Lp = 2^k > L
    const bool plain_io = !padded && a.aligned16;  // activity in aligned 16-byte pieces, none past a cluster's end
    // the bits of this lane's word that are neurons (all of them unless the clusters are padded)
    const uint32_t pmask = !x.valid ? 0u : padded ? pad_mask((uint32_t)a.L, x.gl & kInCluster) : 0xFFFFFFFFu;
    uint32_t v;
    if (a.sym_in) {
        const int32_t *sym = a.sym_in + probe_offset(k0, a.C) + second * a.C;
        v = x.valid ? symbol_word(sym[x.myc], (uint32_t)a.L, x.gl & kInCluster) : 0u;
    } else if (plain_io) {
        const uint4 *p = reinterpret_cast<const uint4 *>(a.V0 + probe_offset(k0, a.n) + (x.valid ? boff : 0u));
        const uint4 lo = p[0], hi = p[1];
        v = x.valid ? (pack16(lo) | (pack16(hi) << 16)) : 0u;
    } else {
        const uint8_t *src = a.V0 + probe_offset(kmine, a.n) + x.myc * (uint32_t)a.L;
        v = x.valid ? load_cluster_word(src, (uint32_t)a.L, x.gl & kInCluster, kmine == a.K - 1 && x.myc == (uint32_t)a.C - 1u) : 0u;
    }

    int it0 = 0, it1 = 0;
    bool done0 = false, done1 = false;
    if (RULE == GBNN_SUM_OF_MAX || RULE == GBNN_HYBRID) {
        // Erased clusters = clusters with no active neuron in the probe.
        const bool erased = x.valid && group_or<LGL>(v) == 0u;
        const uint32_t probe = v;
        uint32_t acc, d;
        bool chg0 = true, chg1 = true;
        if (RULE == GBNN_SUM_OF_MAX) {
            // Section III-C: erased clusters start fully active.  Pass 1: the known clusters contribute
            // the rows of their active neurons, the (fully active) erased clusters their summary rows.
            uint32_t pw = v;
            const uint64_t full = *a.full;  // clusters whose summary row is all ones: it changes nothing, not fetched
            uint64_t summask = ballot(erased && x.islead && !((full >> (x.myc & 63u)) & 1ull));
            if (erased) v = pmask;
            acc = v;
            fetch_and_apply_h<LGL>(x, pw, summask, acc);
            d = acc ^ v;
            const uint64_t dm = ballot(d != 0u);
            chg0 = lo32(dm) != 0u;
            chg1 = hi32(dm) != 0u;
        } else {
            // Algorithm 2, lines 1-5.  A probe keeps the contract (every known cluster holds exactly one
            // active neuron) iff no lane holds two active neurons and as many lanes hold one as there are
            // known clusters.
            const uint32_t pc = __popc(v);
            const uint64_t nz = ballot(pc > 0u), multi = ballot(pc > 1u), knownm = ballot(x.islead && !erased);
            const uint32_t known0 = __popc(lo32(knownm)), known1 = __popc(hi32(knownm));
            const bool contract = multi == 0ull && (uint32_t)__popc(lo32(nz)) == known0 &&
                                  (uint32_t)__popc(hi32(nz)) == known1;
            if (contract) {
                // "exactly C - e signals" then means "adjacent to every known active neuron": the AND of
                // their rows over the erased clusters.
                uint32_t pw = v;
                uint64_t summask = 0;
                acc = erased ? pmask : v;
                fetch_and_apply_h<LGL>(x, pw, summask, acc);
                acc = erased ? acc : v;
                d = erased ? 1u : 0u;  // known clusters have just been applied: clean
            } else {
                // General probes: count the signals, keep the erased-cluster neurons with exactly C - e.
                const uint32_t eq = signals_equal_h(x, v, x.mine(known0, known1));
                acc = erased ? eq : v;
                d = x.valid ? 1u : 0u;
            }
            // the stop test is made only after a bail-out-early pass (Algorithm 2, line 13)
        }
        // When both probes are the usual kind (or finished already) the remaining passes run on the
        // candidates' adjacency matrices; otherwise both take the general loop below.
        bool finished = false;
        if (chg0 || chg1) {
            const uint32_t pcp = __popc(probe);
            const uint64_t nz = ballot(pcp > 0u), multi = ballot(pcp > 1u), knownm = ballot(x.islead && !erased);
            const uint64_t lost = ballot(!erased && acc != probe);
            const uint32_t cand = erased ? acc : 0u;
            const uint64_t bare = ballot(erased && group_or<LGL>(cand) == 0u);
            const uint64_t c1 = ballot(cand != 0u), c2 = ballot((cand & (cand - 1u)) != 0u);
            const bool ok0 = !chg0 || (lo32(multi) == 0u && __popc(lo32(nz)) == __popc(lo32(knownm)) && lo32(lost) == 0u &&
                                       lo32(bare) == 0u && __popc(lo32(c1)) + __popc(lo32(c2)) <= kHalfListMax);
            const bool ok1 = !chg1 || (hi32(multi) == 0u && __popc(hi32(nz)) == __popc(hi32(knownm)) && hi32(lost) == 0u &&
                                       hi32(bare) == 0u && __popc(hi32(c1)) + __popc(hi32(c2)) <= kHalfListMax);
            if (ok0 && ok1) {
                const uint32_t mine_cand = lane_of(halves(chg0, chg1)) ? cand : 0u;
                uint32_t pw = mine_cand, list, T0, T1, first_rank = 0u;
                uint64_t summask = 0;
                take_chunk_h(x, pw, summask, list, T0, T1, &first_rank);
                if (ballot(pw != 0u) == 0ull && (T0 >= 1u || !chg0) && (T1 >= 1u || !chg1)) {
                    candidate_passes_h<RULE, LGL>(x, probe, mine_cand, first_rank, list, T0, T1, chg0, chg1, acc,
                                                  a.max_iters, v, it0, it1);
                    finished = true;
                }
            }
        }
        for (int p = 1; !finished; ++p) {
            v = acc;
            if (!done0 && (!chg0 || p == a.max_iters)) {
                it0 = chg0 ? -p : p;
                done0 = true;
            }
            if (!done1 && (!chg1 || p == a.max_iters)) {
                it1 = chg1 ? -p : p;
                done1 = true;
            }
            if (done0 && done1) break;
            acc = som_step_h<LGL>(x, v, d);  // a probe that is done has d == 0: it lists nothing and keeps v
            if (RULE == GBNN_HYBRID) acc = erased ? acc : v;  // known clusters are frozen
            d = acc ^ v;
            const uint64_t dm = ballot(d != 0u);
            chg0 = lo32(dm) != 0u;
            chg1 = hi32(dm) != 0u;
        }
    } else {
        // Algorithm 1 with Eq. (3)-(5).
        Planes<1> pl;
        pl.hi = sos_hi + (threadIdx.x >> 6) * ((kPlanes - kRegPlanes) * 64) + lane;
        for (int p = 1;; ++p) {
            // a probe that is done lists no rows; its lanes are not updated below
            const bool live = lane_of(halves(!done0, !done1));
            const uint32_t vl = live ? v : 0u;
            const uint32_t rows = count_signals_h(x, vl, pl);
            const unsigned top = rows + (unsigned)a.gamma;
            const int P = top ? 32 - __builtin_clz(top) : 0;
            if (a.gamma) {  // s_i += gamma * v_i : ripple add of a constant into the active neurons
                uint32_t cy = 0u;
#pragma unroll
                for (int q = 0; q < kRegPlanes; ++q) {
                    if (q >= P) break;
                    const uint32_t g = ((a.gamma >> q) & 1) ? vl : 0u;
                    GBNN_FA(pl.lo[q][0], g, cy, pl.lo[q][0], cy);
                }
                for (int q = kRegPlanes; q < P; ++q) {
                    const uint32_t g = ((a.gamma >> q) & 1) ? vl : 0u;
                    uint32_t sum;
                    GBNN_FA(pl.get_hi(q, 0), g, cy, sum, cy);
                    pl.set_hi(q, 0, sum);
                }
                if (P - kRegPlanes > pl.nhi) pl.nhi = P - kRegPlanes;
            }
            // Eq. (4)-(5): per cluster keep the neurons whose score is the cluster maximum, found
            // digit by digit from the top.
            uint32_t cand = pmask;
            for (int q = P - 1; q >= kRegPlanes; --q) {
                const uint32_t tt = cand & pl.get_hi(q, 0);
                if (group_or<LGL>(tt) != 0u) cand = tt;
            }
#pragma unroll
            for (int q = kRegPlanes - 1; q >= 0; --q) {
                if (q >= P) continue;
                const uint32_t tt = cand & pl.lo[q][0];
                if (group_or<LGL>(tt) != 0u) cand = tt;
            }
            cand = live ? cand : v;
            const uint64_t dm = ballot(cand != v);
            const bool chg0 = lo32(dm) != 0u, chg1 = hi32(dm) != 0u;
            v = cand;
            if (!done0 && (!chg0 || p == a.max_iters)) {
                it0 = chg0 ? -p : p;
                done0 = true;
            }
            if (!done1 && (!chg1 || p == a.max_iters)) {
                it1 = chg1 ? -p : p;
                done1 = true;
            }
            if (done0 && done1) break;
        }
    }

    // ---- result store
    if (a.iters && x.gl == 0u && pvalid) a.iters[kmine] = upper ? it1 : it0;
    if (a.sym_in) {
        if (a.bits_out) {
            uint32_t *out = a.bits_out + probe_offset(k0, a.nw) + second * a.nw;  // (this lane's probe)
            if (!padded) {
                if (x.valid) out[x.gl] = v;
            } else if ((a.L & 31) == 0) {
                // whole words: the words of a cluster that exist go to their canonical places
                const uint32_t wi = x.gl & kInCluster;
                if (x.valid && 32u * wi < (uint32_t)a.L) out[x.myc * ((uint32_t)a.L >> 5) + wi] = v;
            } else {
                // clusters share words: the canonical bit vector of each probe is put together in LDS
                uint32_t *canon = lds_words + (threadIdx.x >> 6) * (kLdsWords / 4) + (upper ? 32u : 0u);
                if (x.gl < (uint32_t)a.nw) canon[x.gl] = 0u;
                wave_lds_sync();
                if (x.valid) or_cluster_word(canon, x.myc, (uint32_t)a.L, x.gl & kInCluster, v);
                wave_lds_sync();
                if (pvalid && x.gl < (uint32_t)a.nw) out[x.gl] = canon[x.gl];
            }
        }
        if (a.sym_out) {
            const int32_t sy = cluster_symbol<LGL>(v, x.gl & kInCluster);
            if (x.islead) a.sym_out[probe_offset(k0, a.C) + second * a.C + x.myc] = sy;
        }
    } else if (plain_io) {
        // A half's words are 32 nw bytes: written as two contiguous pieces, lane j of the half storing 16 bytes at
        // 16 j of each -- half (j & 1) of the word of lane j / 2 (first piece) and of lane 16 + j / 2 (second
        // piece) -- so that every store instruction covers whole lines; non-temporal, as the results are not
        // read again and should not displace the table and the probes in the caches.
        const uint32_t wa = entry(v, x.basev + ((x.gl >> 1) << 2));
        const uint32_t wb = entry(v, x.basev + ((16u + (x.gl >> 1)) << 2));
        const uint32_t sh = (x.gl & 1u) * 16u;
        uint8_t *piece = a.Vout + probe_offset(k0, a.n) + (upper ? (uint32_t)a.n : 0u) + 16u * x.gl;
        if (pvalid && (x.gl >> 1) < (uint32_t)a.nw) store16_nontemporal(piece, spread16((wa >> sh) & 0xFFFFu));
        if (pvalid && 16u + (x.gl >> 1) < (uint32_t)a.nw) store16_nontemporal(piece + 512, spread16((wb >> sh) & 0xFFFFu));
    } else {
        // Padded clusters, or buffers that are not 16-byte aligned: each half puts its canonical bit vector together
        // in LDS and writes the n bytes of its result front to back, 16 bytes per lane and step at whatever
        // alignment the result has (non-temporal as above); the last n mod 16 bytes one by one.
        uint32_t *canon = lds_words + (threadIdx.x >> 6) * (kLdsWords / 4) + (upper ? 32u : 0u);
        if (x.gl < (uint32_t)a.nw) canon[x.gl] = 0u;
        wave_lds_sync();
        if (x.valid) or_cluster_word(canon, x.myc, (uint32_t)a.L, x.gl & kInCluster, v);
        wave_lds_sync();
        if (pvalid) {
            uint8_t *dstb = a.Vout + probe_offset(kmine, a.n);
            const uint16_t *canon16 = reinterpret_cast<const uint16_t *>(canon);
            const uint32_t pieces = (uint32_t)a.n >> 4;
            for (uint32_t j = x.gl; j < pieces; j += 32u) store16_unaligned_nontemporal(dstb + 16u * j, spread16(canon16[j]));
            const uint32_t i = (pieces << 4) + x.gl;
            if (x.gl < ((uint32_t)a.n & 15u)) dstb[i] = (uint8_t)((canon[i >> 5] >> (i & 31u)) & 1u);
        }
    }
}

template <int LGL>
hipError_t launch_one_h(const RetrieveArgs &a, hipStream_t s)
{
    const int wpb = 4;
    const int64_t pairs = (a.K + 1) / 2;
    const int64_t blocks = (pairs + wpb - 1) / wpb;
    const dim3 grid((unsigned)blocks), block(64 * wpb);
    switch (a.rule) {
    case GBNN_SUM_OF_SUM:
        hipLaunchKernelGGL((k_retrieve_half<GBNN_SUM_OF_SUM, LGL>), grid, block, 0, s, a);
        break;
    case GBNN_SUM_OF_MAX:
        hipLaunchKernelGGL((k_retrieve_half<GBNN_SUM_OF_MAX, LGL>), grid, block, 0, s, a);
        break;
    default:
        hipLaunchKernelGGL((k_retrieve_half<GBNN_HYBRID, LGL>), grid, block, 0, s, a);
        break;
    }
    return hipGetLastError();
}

}  // namespace

// Shapes served: L a power of two >= 32 and at most 32 packed words per probe.
bool half_wave_serves(int C, int L)
{
    const Geometry g = geometry(C, L);  // (clusters padded to a power of two of at least 32 neurons)
    if (g.Lp < 32 || (g.Lp & (g.Lp - 1)) != 0 || g.Lp < L) return false;
    return g.nwp <= 32;
}

hipError_t launch_retrieve_half(const RetrieveArgs &a, hipStream_t s)
{
    if (a.K == 0) return hipSuccess;
    if (!half_wave_serves(a.C, a.L)) return hipErrorInvalidValue;
    switch (a.Lp / 32) {  // lanes per cluster; C >= 2 keeps it at 16 or below
    case 1: return launch_one_h<0>(a, s);
    case 2: return launch_one_h<1>(a, s);
    case 4: return launch_one_h<2>(a, s);
    case 8: return launch_one_h<3>(a, s);
    case 16: return launch_one_h<4>(a, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace gbnn
