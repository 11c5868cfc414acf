// Internal declarations shared by the host entry points and the kernel launchers.
// Not part of the public interface (that is include/gbnn.h).
#ifndef GBNN_INTERNAL_H
#define GBNN_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gbnn.h"

namespace gbnn {

// How the kernels see the clusters of a network.  The register kernels hold a cluster in 2^k consecutive
// lanes, i.e. they need clusters of Lp = 2^k >= 32 neurons; a network whose L is not such a number is
// padded for them: cluster c occupies neurons c*Lp .. c*Lp + L - 1 of a padded network of np = C*Lp
// neurons, the other neurons of a padded cluster do not exist (never on, no edges).  The prepared table
// is laid out for the padded network; W, activity vectors and packed results at the interface keep the
// canonical layout.  Shapes that no register kernel serves (Lp > 2048 or np beyond the interface's limit)
// are not padded: the any-shape kernel reads the canonical layout.
struct Geometry {
    int Lp, np, nwp;  // neurons per padded cluster, padded neurons, words per row of the prepared table
    bool padded;      // Lp != L
};
inline Geometry geometry(int C, int L)
{
    int Lp = 32;
    while (Lp < L) Lp <<= 1;
    if (Lp <= 2048 && (int64_t)C * Lp <= GBNN_MAX_N) return Geometry{Lp, C * Lp, C * Lp / 32, Lp != L};
    return Geometry{L, C * L, (C * L + 31) / 32, false};
}

// Arguments of one retrieval launch; all pointers are device pointers.
struct RetrieveArgs {
    const uint32_t *W;    // canonical adjacency, uint32[n][nw]
    const uint32_t *Wb;   // the prepared table, uint32[np + C + 2][nwp]: W with all-one intra-cluster blocks, followed directly by
    const uint32_t *has;  // the cluster summaries, uint32[C][nwp]: bit i of row c' = "i is in c' or adjacent to a neuron of c'"
    const uint32_t *hasc; // the same summaries in the canonical layout, uint32[C][nw] (= has when nothing is padded)
    const uint64_t *full; // one word: bit c' set = the summary row of c' is all ones (ANDing it changes nothing)
    const uint8_t *V0;    // uint8[K][n]                       } the activity boundary (gbnn_retrieve);
    uint8_t *Vout;        // uint8[K][n]                       } both nullptr at the message boundary
    const int32_t *sym_in;  // int32[K][C] or nullptr: the message boundary (gbnn_retrieve_symbols) when set
    uint32_t *bits_out;     // uint32[K][nw] or nullptr        } outputs of the message boundary
    int32_t *sym_out;       // int32[K][C] or nullptr          }
    int32_t *iters;       // int32[K] or nullptr
    int64_t K;
    int C, L, n, nw;      // the network as the interface sees it
    int Lp, np, nwp;      // ... and as the register kernels do (geometry())
    bool aligned16;       // V0, Vout and L are all multiples of 16 (activity boundary)
    bool stream_in;       // read the probes with streaming loads (see retrieve_common)
    int rule, gamma, max_iters;
};

// Workspace layout: one table of np + C + 2 rows of nwp words.  Rows 0..np-1: W (padded layout) with all-one
// intra-cluster blocks; rows np..np+C-1: the cluster summaries; row np+C: all zero and row np+C+1: all ones
// (what the padding entries of a batch of row fetches read when rows are counted, resp. ANDed).  One table,
// so that one buffer resource reaches all of it.
constexpr int kTableExtraRows = 2;  // the all-zero and the all-one row
inline size_t workspace_has_offset(int C, int L)
{
    const Geometry g = geometry(C, L);
    return (size_t)g.np * g.nwp * sizeof(uint32_t);
}
// ... followed, at the next multiple of 256 bytes, by 256 bytes of flags: one uint64, bit c set = summary row
// c is all ones (the rest zero) ...
inline size_t workspace_full_offset(int C, int L)
{
    const Geometry g = geometry(C, L);
    return (((size_t)g.np + C + kTableExtraRows) * g.nwp * sizeof(uint32_t) + 255) & ~(size_t)255;
}
// ... and, for a padded network, by the cluster summaries in the canonical layout, uint32[C][nw] (what the
// any-shape kernel reads), rounded up to 256 bytes.
inline size_t workspace_canonical_offset(int C, int L) { return workspace_full_offset(C, L) + 256; }
inline size_t workspace_total_bytes(int C, int L)
{
    const Geometry g = geometry(C, L);
    const size_t extra = g.padded ? (((size_t)C * ((C * L + 31) / 32) * sizeof(uint32_t) + 255) & ~(size_t)255) : 0;
    return workspace_canonical_offset(C, L) + extra;
}

// Which kernel family serves a shape.  One wavefront per probe: packed words per lane (1, 2, 4, 8),
// 0 = not served.  Half a wavefront per probe (two probes per wave, one word
// per lane): yes or no.
int wave_words_per_lane(int C, int L);
bool half_wave_serves(int C, int L);

// Which storing kernel: chosen by the number of messages, or forced (tests).
enum { kStoreAuto = 0, kStoreAtomic = 1, kStoreRows = 2 };
constexpr int64_t kStoreRowsMinMessages = 64;
constexpr int kStoreBlocks = 256;
hipError_t launch_store(uint32_t *W, int C, int L, int nw, const int32_t *msgs, int64_t M, int32_t *status,
                        int path, hipStream_t s);
// Both take the workspace (workspace_*_offset above say where its parts are).
hipError_t launch_store_update(uint32_t *W, int C, int L, int nw, const int32_t *msgs, int64_t M, int32_t *status,
                               char *workspace, hipStream_t s);
hipError_t launch_prepare(const uint32_t *W, int C, int L, int nw, char *workspace, hipStream_t s);
// The cluster summaries of W (canonical layout) and the flags "row c is all ones" (part of gbnn_sparsify).
hipError_t launch_summary(const uint32_t *W, int C, int L, int nw, uint32_t *has, uint64_t *full, hipStream_t s);

// Sparse W': byte offsets of its parts (offsets at 0), and the launchers.
size_t sparse_summary_offset(int n);
size_t sparse_full_offset(int C, int n, int nw);
size_t sparse_cols_offset(int C, int n, int nw);
hipError_t launch_sparse_count(const uint32_t *W, int n, int nw, unsigned long long *total, hipStream_t s);
hipError_t launch_sparsify(const uint32_t *W, int C, int L, int nw, char *Wp, size_t Wp_bytes, int32_t *status,
                           hipStream_t s);
hipError_t launch_retrieve_sparse(const char *Wp, size_t Wp_bytes, int C, int L, int nw, const int32_t *probes,
                                  int64_t K, int max_iters, uint32_t *bits_out, int32_t *sym_out, int32_t *iters,
                                  hipStream_t s);

hipError_t launch_retrieve_wave(const RetrieveArgs &a, int words_per_lane, hipStream_t s);
hipError_t launch_retrieve_half(const RetrieveArgs &a, hipStream_t s);
hipError_t launch_retrieve_generic(const RetrieveArgs &a, hipStream_t s);

}  // namespace gbnn
#endif
