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
    const uint32_t *has;  // cluster summaries, uint32[C][nw]: bit i of row c' = "some neuron of c' is adjacent to i"
    const uint8_t *V0;    // uint8[K][n]
    uint8_t *Vout;        // uint8[K][n]
    int32_t *iters;       // int32[K] or nullptr
    int64_t K;
    int C, L, n, nw;
    int rule, gamma, max_iters;
};

// Byte offset / size of the cluster-summary table inside the caller's workspace.
inline size_t workspace_has_bytes(int C, int nw) { return (size_t)C * (size_t)nw * sizeof(uint32_t); }

// Which kernel family serves a shape: 0 = generic, otherwise packed words per lane (1, 2, 4).
int wave_words_per_lane(int C, int L);

hipError_t launch_store(uint32_t *W, int C, int L, int nw, const int32_t *msgs, int64_t M, int32_t *status,
                        hipStream_t s);
hipError_t launch_cluster_summary(const uint32_t *W, int C, int L, int nw, uint32_t *has, hipStream_t s);
hipError_t launch_retrieve_wave(const RetrieveArgs &a, int words_per_lane, hipStream_t s);
hipError_t launch_retrieve_generic(const RetrieveArgs &a, hipStream_t s);

}  // namespace gbnn
#endif
