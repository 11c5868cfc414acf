// Internal declarations shared by the host entry points and the kernel launchers.
// Not part of the public interface (that is include/gbnn.h).
#ifndef GBNN_INTERNAL_H
#define GBNN_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gbnn.h"

namespace gbnn {

// Arguments of one retrieval launch; all pointers are device pointers.
struct RetrieveArgs {
    const uint32_t *W;    // canonical adjacency, uint32[n][nw]
    const uint32_t *Wb;   // W with all-one intra-cluster blocks, uint32[n][nw], followed directly by
    const uint32_t *has;  // the cluster summaries, uint32[C][nw]: bit i of row c' = "i is in c' or adjacent to a neuron of c'"
    const uint64_t *full; // one word: bit c' set = the summary row of c' is all ones (ANDing it changes nothing)
    const uint8_t *V0;    // uint8[K][n]                       } the activity boundary (gbnn_retrieve);
    uint8_t *Vout;        // uint8[K][n]                       } both nullptr at the message boundary
    const int32_t *sym_in;  // int32[K][C] or nullptr: the message boundary (gbnn_retrieve_symbols) when set
    uint32_t *bits_out;     // uint32[K][nw] or nullptr        } outputs of the message boundary
    int32_t *sym_out;       // int32[K][C] or nullptr          }
    int32_t *iters;       // int32[K] or nullptr
    int64_t K;
    int C, L, n, nw;
    int rule, gamma, max_iters;
};

// Workspace layout: one table of n + C + 2 rows of nw words.  Rows 0..n-1: W with all-one intra-cluster
// blocks; rows n..n+C-1: the cluster summaries; row n+C: all zero and row n+C+1: all ones (what the
// padding entries of a batch of row fetches read when rows are counted, resp. ANDed).  One table, so
// that one buffer resource reaches all of it.
constexpr int kTableExtraRows = 2;  // the all-zero and the all-one row
inline size_t workspace_has_offset(int C, int L, int nw) { return (size_t)C * L * nw * sizeof(uint32_t); }
// ... followed, at the next multiple of 256 bytes, by one uint64: bit c set = summary row c is all ones.
inline size_t workspace_full_offset(int C, int L, int nw)
{
    return (((size_t)C * L + C + kTableExtraRows) * nw * sizeof(uint32_t) + 255) & ~(size_t)255;
}
inline size_t workspace_total_bytes(int C, int L, int nw) { return workspace_full_offset(C, L, nw) + 256; }

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
hipError_t launch_store_update(uint32_t *W, int C, int L, int nw, const int32_t *msgs, int64_t M, int32_t *status,
                               uint32_t *has, uint32_t *Wb, uint64_t *full, hipStream_t s);
hipError_t launch_prepare(const uint32_t *W, int C, int L, int nw, uint32_t *has, uint32_t *Wb, uint64_t *full,
                          hipStream_t s);
// The cluster summaries of W and the flags "row c is all ones" (part of gbnn_prepare and of gbnn_sparsify).
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
